"""A seeded sweep of ragged batches against the fp64 oracle: lengths around the tile sizes (0, 1, 63..65, 127..129, 255..257
and random ones), every model width the MFMA kernels have instances for, both attention kinds, both attention
configurations, hot inputs.  Complements the fixed stress cases: the same bars, shapes nobody chose by hand."""
import numpy as np
import pytest

import oracle
from paper_2509_22681_amd import workloads as W
from tests.test_gpu_parity import TOL_HOT, score_err

pytestmark = pytest.mark.gpu

EDGE = [0, 1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 192, 255, 256, 257, 383, 511, 512, 513]
MODELS = [(64, 2), (128, 2), (128, 4), (192, 3), (256, 4), (256, 8), (384, 6), (512, 8), (512, 16)]


def draw_case(seed):
    rng = np.random.default_rng(1000 + seed)
    d, H = MODELS[seed % len(MODELS)]
    B = int(rng.integers(1, 6))
    pick = lambda: int(rng.choice(EDGE)) if rng.random() < 0.6 else int(rng.integers(0, 700))
    L = [pick() for _ in range(B)]
    M = [pick() // (1 if rng.random() < 0.5 else 4) for _ in range(B)]
    if sum(M) == 0:
        M[0] = 1 + int(rng.integers(0, 70))
    nb = int(rng.choice([16, 32, 128]))
    D = int(rng.choice([128, 256, 1024]))          # D below the longest history: distances clamp
    return dict(L=L, M=M, d=d, H=H, nb=nb, D=D, layers=int(rng.integers(1, 4)), attn_scale=float(rng.choice([1.0, 0.5, 0.3])),
                kind="softmax" if seed % 3 == 2 else "silu", dtype="f32" if seed % 5 == 4 else "bf16", latency_mode=int(seed % 2))


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2509_22681_amd import binding
    return binding


@pytest.mark.parametrize("seed", range(36))
def test_random_ragged_batch(B, seed):
    import torch
    c = draw_case(seed)
    wl = W.make_custom(c["L"], c["M"], d=c["d"], H=c["H"], n_layers=c["layers"], n_buckets=c["nb"], max_rel_dist=c["D"],
                       dtype=c["dtype"], seed=seed, emb_std=1.0, rab_std=1.0, bias_amp=0.1, affine_random=True,
                       attn_scale=c["attn_scale"], attn_kind=c["kind"], name=f"rand{seed}")
    want = oracle.forward(wl.cfg.to_dict(), wl.weights, wl.history_emb, wl.history_offsets, wl.cand_emb, wl.cand_offsets)
    h = B.flame_gr_create(B.config_for(wl, latency_mode=c["latency_mode"]))
    try:
        dw, hist, cand = B.to_device(wl)
        out = torch.full((int(wl.cand_offsets[-1]),), float("nan"), device="cuda:0")
        B.flame_gr_forward(h, dw, hist, wl.history_offsets, cand, wl.cand_offsets, out)
        torch.cuda.synchronize()
        g = out.cpu().numpy()
    finally:
        B.flame_gr_destroy(h)
    assert np.isfinite(g).all(), c
    # the gate over the whole batch's scores (a request with one or two candidates has no rms of its own to hold a score
    # near zero against)
    worst = score_err(g, want)
    print(f"seed {seed}: {c}: score error {worst:.3e}")
    assert worst <= TOL_HOT[c["dtype"]], (c, worst)


@pytest.mark.parametrize("seed", range(100, 118))
def test_every_way_of_running_a_batch_gives_the_same_bits(B, seed):
    """The same seeded ragged batches through the other entry points and configurations: a captured graph replayed,
    history prefill + candidate scoring, the static-workspace forward, stream groups, and requests split by
    max_seq_tokens.  None of them changes an operand or the order of a sum: every one must equal the plain forward bit
    for bit (SiLU attention; for softmax the split of a request regroups the normalisation and is left out)."""
    import torch
    from tests.test_gpu_two_stage import two_stage
    c = draw_case(seed)
    c["latency_mode"] = 0
    wl = W.make_custom(c["L"], c["M"], d=c["d"], H=c["H"], n_layers=c["layers"], n_buckets=c["nb"], max_rel_dist=c["D"],
                       dtype=c["dtype"], seed=seed, emb_std=1.0, rab_std=1.0, bias_amp=0.1, affine_random=True,
                       attn_scale=c["attn_scale"], attn_kind=c["kind"], name=f"ways{seed}")
    n = int(wl.cand_offsets[-1])
    dw, hist, cand = B.to_device(wl)

    def forward(**kw):
        grow = kw.pop("grow", False)
        cfg = B.config_for(wl, **kw)
        if grow:                                   # splitting repeats histories: room for the copies
            cfg.max_total_tokens = int(cfg.max_total_tokens * 8 + 1024)
            cfg.max_requests = int(cfg.max_requests * 16 + 16)
        h = B.flame_gr_create(cfg)
        try:
            out = torch.full((n,), float("nan"), device="cuda:0")
            B.flame_gr_forward(h, dw, hist, wl.history_offsets, cand, wl.cand_offsets, out)
            torch.cuda.synchronize()
            return out.cpu().numpy().copy()
        finally:
            B.flame_gr_destroy(h)

    ref = forward()
    assert np.isfinite(ref).all()
    ways = {"stream groups": forward(n_streams=3)}
    # a captured graph, replayed twice
    h = B.flame_gr_create(B.config_for(wl))
    try:
        out = torch.zeros(n, device="cuda:0")
        B.flame_gr_capture(h, dw, hist, wl.history_offsets, cand, wl.cand_offsets, out)
        for rep in range(2):
            out.fill_(float("nan"))
            B.flame_gr_replay(h)
            torch.cuda.synchronize()
            ways[f"graph replay {rep}"] = out.cpu().numpy().copy()
    finally:
        B.flame_gr_destroy(h)
    if c["dtype"] == "bf16":                      # the two-stage path is built for the MFMA kernels only
        (ways["prefill + score"],) = two_stage(B, wl)
    out = torch.full((n,), float("nan"), device="cuda:0")
    B.flame_gr_forward_static(B.config_for(wl), dw, hist, wl.history_offsets, cand, wl.cand_offsets, out)
    torch.cuda.synchronize()
    ways["static workspace"] = out.cpu().numpy().copy()
    if c["kind"] == "silu" and max(c["L"]) + 1 <= 400 and max(c["M"]) > 3:
        ways["split by max_seq_tokens"] = forward(max_seq_tokens=max(c["L"]) + max(2, max(c["M"]) // 3), grow=True)
    for name, g in ways.items():
        assert np.array_equal(g, ref), (name, c, float(np.nanmax(np.abs(g - ref))))
    print(f"seed {seed}: {sorted(ways)} equal the plain forward on {c}")
