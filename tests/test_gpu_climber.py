"""GPU parity of the sub-sequence blocks + gating fusion + task head path (the paper's own model, Section 2.1, in the
reading of include/flame_climber.h) against the fp64 CPU oracle."""
import numpy as np
import pytest

import oracle
from paper_2509_22681_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2509_22681_amd import binding
    return binding


def head_weights(nb, d, T, E, seed):
    rng = np.random.default_rng(seed)
    return dict(wg=(rng.standard_normal((nb, d, nb * d)) / np.sqrt(nb * d)).astype(np.float32),
                cg=(rng.standard_normal((nb, d)) * 0.3).astype(np.float32),
                a_w=(rng.standard_normal((T, E, d)) / np.sqrt(d)).astype(np.float32),
                a_b=(rng.standard_normal((T, E)) * 0.2).astype(np.float32),
                v=(rng.standard_normal((T, E)) / np.sqrt(E)).astype(np.float32),
                c=(rng.standard_normal(T) * 0.2).astype(np.float32))


def make_model(L, M, n_blocks, *, d, H, layers, dtype, seed, hot):
    """One batch of requests and n_blocks weight sets (softmax attention); block b gets its own seed."""
    kw = dict(emb_std=1.0, rab_std=1.0, bias_amp=0.1, affine_random=True) if hot else {}
    wls = [W.make_custom(L, M, d=d, H=H, n_layers=layers, n_buckets=16, max_rel_dist=1024, dtype=dtype, seed=seed + 17 * b,
                         attn_kind="softmax", name=f"block{b}", **kw) for b in range(n_blocks)]
    return wls[0], [w.weights for w in wls]


def block_batch(base, n_blocks, b):
    """The jagged batch block b sees: slice b of every request's history, all candidates."""
    ho = base.history_offsets
    parts, lens = [], []
    for i in range(base.n_requests):
        sl = oracle.block_slices(int(ho[i + 1] - ho[i]), n_blocks)[b]
        parts.append(base.history_emb[ho[i] + sl.start:ho[i] + sl.stop])
        lens.append(sl.stop - sl.start)
    hist = np.concatenate(parts, 0) if parts else np.zeros((0, base.cfg.d_model), np.float32)
    return hist, np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)


def climber_gpu(B, base, block_weights, head):
    import torch
    nb = len(block_weights)
    n = int(base.cand_offsets[-1])
    d = base.cfg.d_model
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.float32)).to("cuda:0")
    hidden, handles = [], []
    try:
        for b in range(nb):
            hist, ho = block_batch(base, nb, b)
            wl = W.Workload(f"b{b}", base.cfg, ho, base.cand_offsets, hist, base.cand_emb, block_weights[b])
            h = B.flame_gr_create(B.config_for(wl))
            handles.append(h)
            dw, dh, dc = B.to_device(wl)
            out = torch.full((n, d), float("nan"), device="cuda:0", dtype=torch.float32)
            B.flame_gr_forward_hidden(h, dw, dh, ho, dc, base.cand_offsets, out)
            hidden.append(out)
        head_dev = {k: dev(v) for k, v in head.items()}
        fused = torch.empty((n, d), device="cuda:0", dtype=torch.float32)
        probs = torch.full((n, len(head["c"])), float("nan"), device="cuda:0", dtype=torch.float32)
        B.flame_climber_head(head_dev, hidden, fused, probs)
        torch.cuda.synchronize()
        return probs.cpu().numpy()
    finally:
        for h in handles:
            B.flame_gr_destroy(h)


def climber_oracle(base, block_weights, head):
    cfg = base.cfg.to_dict()
    ho, co = base.history_offsets, base.cand_offsets
    return np.concatenate([oracle.climber_request(cfg, block_weights, head, base.history_emb[ho[i]:ho[i + 1]],
                                                  base.cand_emb[co[i]:co[i + 1]]) for i in range(base.n_requests)], 0)


def test_head_alone_on_ragged_shapes(B):
    import torch
    rng = np.random.default_rng(4)
    for nb, d, T, E, rows in [(3, 40, 3, 70, 131), (1, 64, 1, 1, 1), (2, 128, 2, 256, 700), (8, 8, 5, 9, 65),
                              (2, 192, 2, 160, 97), (2, 36, 2, 33, 70), (3, 12, 1, 130, 33)]:
        Hs = [rng.standard_normal((rows, d)).astype(np.float32) * 1.5 for _ in range(nb)]
        hw = head_weights(nb, d, T, E, nb)
        want = oracle.fuse_and_score(hw, Hs)
        dev = lambda a: torch.from_numpy(a).to("cuda:0")
        fused = torch.empty((rows, d), device="cuda:0")
        probs = torch.full((rows, T), float("nan"), device="cuda:0")
        B.flame_climber_head({k: dev(v) for k, v in hw.items()}, [dev(h) for h in Hs], fused, probs)
        torch.cuda.synchronize()
        err = np.abs(probs.cpu().numpy() - want).max()
        assert err <= 2e-6, (nb, d, T, E, rows, err)
    # hidden rows that are not 16-byte aligned take the kernels that load single floats: same result
    nb, d, T, E, rows = 2, 64, 2, 48, 77
    Hs = [rng.standard_normal((rows, d)).astype(np.float32) for _ in range(nb)]
    hw = head_weights(nb, d, T, E, 5)
    want = oracle.fuse_and_score(hw, Hs)
    shifted = []
    for h_ in Hs:
        buf = torch.zeros(rows * d + 1, device="cuda:0")
        buf[1:] = dev(h_).reshape(-1)
        shifted.append(buf[1:].view(rows, d))
        assert shifted[-1].data_ptr() % 16 == 4
    fused = torch.empty((rows, d), device="cuda:0")
    probs = torch.full((rows, T), float("nan"), device="cuda:0")
    B.flame_climber_head({k: dev(v) for k, v in hw.items()}, shifted, fused, probs)
    torch.cuda.synchronize()
    assert np.abs(probs.cpu().numpy() - want).max() <= 2e-6
    # error paths: no blocks, too many blocks, a missing weight
    hw = {k: dev(v) for k, v in head_weights(1, 8, 1, 2, 0).items()}
    h1 = torch.zeros((4, 8), device="cuda:0")
    with pytest.raises(B.FlameGRError) as e:
        B.flame_climber_head(hw, [h1] * 9, torch.empty((4, 8), device="cuda:0"), torch.empty((4, 1), device="cuda:0"))
    assert e.value.code == -1
    with pytest.raises(B.FlameGRError) as e:
        B.flame_climber_head(dict(hw, v=None), [h1], torch.empty((4, 8), device="cuda:0"), torch.empty((4, 1), device="cuda:0"))
    assert e.value.code == -1


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n_blocks", [1, 2, 3])
def test_blocks_fusion_head_against_the_oracle(B, dtype, n_blocks):
    base, bw = make_model([150, 64, 0, 301, 5], [70, 128, 9, 40, 3], n_blocks, d=128, H=2, layers=2, dtype=dtype, seed=3, hot=True)
    head = head_weights(n_blocks, 128, 3, 96, 11)
    g = climber_gpu(B, base, bw, head)
    o = climber_oracle(base, bw, head)
    assert np.isfinite(g).all() and g.shape == o.shape
    err = float(np.abs(g - o).max())
    print(f"{n_blocks} blocks, {dtype}: max |p_gpu - p_oracle| = {err:.3e}")
    # probabilities: absolute error.  fp32 path 1e-4; fp16 path 2e-2 (the bar of the scores, a logistic function
    # has slope <= 1/4, the residual rows feeding it are O(1))
    assert err <= (1e-4 if dtype == "f32" else 2e-2), err


def test_paper_base_scenario_shape(B):
    """Table 2's base scenario (sequence 512, 128 candidates, 2 blocks x 12 layers) at cool, benchmark-like values."""
    base, bw = make_model([512] * 4, [128] * 4, 2, d=128, H=2, layers=12, dtype="bf16", seed=5, hot=False)
    head = head_weights(2, 128, 2, 128, 13)
    g = climber_gpu(B, base, bw, head)
    o = climber_oracle(base, bw, head)
    err = float(np.abs(g - o).max())
    print(f"base scenario (512 + 128, 2 x 12 layers): max |p_gpu - p_oracle| = {err:.3e}")
    assert err <= 2e-2
