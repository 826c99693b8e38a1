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
