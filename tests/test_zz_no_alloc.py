"""flame_gr_forward_static: the forward in the library's static device workspace, for callers that cannot allocate.

Its scores must equal those of flame_gr_forward (a handle with its own workspaces) on the same inputs bit for bit:
the kernels and their launch shapes are the same, only where the workspaces live differs.  Calls follow one another
on one GPU with different models, element types and sizes, so every call finds the array filled by a call of another
layout, and the later ones are smaller than the first."""
import numpy as np
import pytest

from paper_2509_22681_amd import workloads as W


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2509_22681_amd import binding
    return binding


def handle_scores(B, wl, **kw):
    import torch
    h = B.flame_gr_create(B.config_for(wl, **kw))
    try:
        dw, hist, cand = B.to_device(wl)
        out = torch.full((int(wl.cand_offsets[-1]),), float("nan"), device="cuda:0", dtype=torch.float32)
        B.flame_gr_forward(h, dw, hist, wl.history_offsets, cand, wl.cand_offsets, out)
        torch.cuda.synchronize()
        return out.cpu().numpy()
    finally:
        B.flame_gr_destroy(h)


def static_scores(B, wl, **kw):
    import torch
    dw, hist, cand = B.to_device(wl)
    out = torch.full((int(wl.cand_offsets[-1]),), float("nan"), device="cuda:0", dtype=torch.float32)
    cfg = B.config_for(wl, **kw)
    cfg.max_requests = 0            # the capacity fields are ignored by this entry point
    cfg.max_total_tokens = 0
    B.flame_gr_forward_static(cfg, dw, hist, wl.history_offsets, cand, wl.cand_offsets, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def hot(L, M, d, H, dtype, layers=2, nb=16, D=None, seed=3, kind="silu"):
    return W.make_custom(L, M, d=d, H=H, n_layers=layers, n_buckets=nb, max_rel_dist=D, dtype=dtype, seed=seed, emb_std=1.0,
                         rab_std=1.0, bias_amp=0.1, affine_random=True, attn_kind=kind, name="static")


@pytest.mark.gpu
def test_static_workspace_forward_equals_the_handle_forward(B):
    calls = [
        # a batch of several ragged requests, fused output projection (d = 128)
        (hot([700, 65, 0, 129], [130, 257, 5, 1], 128, 2, "bf16", D=1024), {}),
        # smaller, another model width (unfused LayerNorm-gate path), latency configuration: its 128-key tiles read
        # the spare rows behind the batch, where the previous call left its data
        (hot([190], [0], 64, 1, "bf16", D=256, seed=4), dict(latency_mode=1)),
        (hot([191, 3], [2, 60], 64, 1, "bf16", D=256, seed=4), dict(latency_mode=1)),
        # fp32 path in the same array
        (hot([64, 10], [16, 3], 64, 2, "f32", nb=128, D=128, seed=5), {}),
        # softmax variant, head width 32
        (hot([150, 64], [70, 128], 256, 8, "bf16", layers=3, D=256, seed=6, kind="softmax"), {}),
        # requests split by candidates (max_seq_tokens)
        (hot([100, 20], [300, 40], 128, 2, "bf16", D=128, seed=7), dict(max_seq_tokens=160, slack_requests=8, slack_tokens=2000)),
        # the first batch again: the array now holds five other layouts
        (hot([700, 65, 0, 129], [130, 257, 5, 1], 128, 2, "bf16", D=1024), {}),
    ]
    for n, (wl, kw) in enumerate(calls):
        got = static_scores(B, wl, **kw)
        want = handle_scores(B, wl, **kw)
        assert np.isfinite(want).all()
        assert np.array_equal(got, want), (n, float(np.max(np.abs(got - want))) if got.size else 0.0)


@pytest.mark.gpu
def test_static_workspace_holds_one_request_of_the_production_model(B):
    wl = W.make_custom([1024], [512], d=512, H=8, n_layers=16, n_buckets=128, max_rel_dist=2048, dtype="bf16", seed=9,
                       name="static_prod")
    cfg = B.config_for(wl)
    need = B.flame_gr_static_scratch_bytes(cfg, 1024 + 512)
    assert need <= 64 << 20, need
    got = static_scores(B, wl)
    assert np.array_equal(got, handle_scores(B, wl))
    # twice as many tokens do not fit: rejected, with both sizes in the message, and nothing runs
    big = W.make_custom([4096], [2000], d=512, H=8, n_layers=16, n_buckets=128, max_rel_dist=8192, dtype="bf16", seed=9,
                        emb_std=0.0, name="static_big")
    with pytest.raises(B.FlameGRError) as e:
        static_scores(B, big)
    assert e.value.code == -2 and "static workspace holds 67108864" in str(e.value)
    assert np.array_equal(static_scores(B, wl), got)


def test_static_workspace_size_check_needs_no_gpu():
    """The size check is host arithmetic that runs before any HIP call: a batch beyond the static array is rejected
    with CAPACITY_EXCEEDED also where there is no GPU (the pointers below are never dereferenced)."""
    from paper_2509_22681_amd import binding as B
    cfg = B.make_config(16, 512, 8, 128, 8192, "bf16")
    rows = 4096 + 2048
    need = B.flame_gr_static_scratch_bytes(cfg, rows)
    # residual pair 4d + four planes and output 10d per row, 256 spare rows; 10 d^2 per layer of weights; bias tables
    d, Ly = 512, 16
    assert need >= (rows + 256) * 14 * d + Ly * 10 * d * d + Ly * 8 * 8192 * 4
    assert need > 64 << 20
    fake = np.zeros(64, np.float32)                      # aligned, non-NULL stand-ins
    w = B.flame_gr_weights(*([fake.ctypes.data] * 8), 0.0, fake.ctypes.data)
    ho, co = np.array([0, 4096], np.int32), np.array([0, 2000], np.int32)
    rc = B._lib.flame_gr_forward_static(cfg, w, fake.ctypes.data, ho.ctypes.data_as(B._i32p), fake.ctypes.data,
                                        co.ctypes.data_as(B._i32p), 1, fake.ctypes.data, None)
    assert rc == -2
    assert "static workspace holds" in B.flame_gr_last_error()
    small = B.flame_gr_static_scratch_bytes(B.make_config(2, 128, 2, 16, 1024, "bf16"), 1536)
    assert small < 8 << 20
