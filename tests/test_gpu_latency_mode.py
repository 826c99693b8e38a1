"""GPU parity of the latency configuration of the MFMA attention kernel (flame_gr_config.latency_mode = 1: pairs
of wavefronts split the keys of every tile) against the fp64 oracle, for both attention kinds, and its own
determinism and batch independence.  Its sums are grouped differently from the throughput configuration, so the
two are compared to rounding only."""
import numpy as np
import pytest

from paper_2509_22681_amd import workloads as W
from tests.oracle_cache import request_scores, sample_requests
from tests.test_gpu_parity import STRESS, TOL, TOL_HOT, oracle_all, score_err, stress
from tests.test_gpu_softmax import gpu_out, oracle_out, soft

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2509_22681_amd import binding
    return binding


@pytest.mark.parametrize("case", list(STRESS))
@pytest.mark.parametrize("kind", ["silu", "softmax"])
def test_latency_mode_against_the_oracle(B, case, kind):
    if kind == "silu":
        wl = stress(dtype="bf16", name=case, hot=True, **STRESS[case])
        want = oracle_all(wl)
    else:
        wl = soft(dtype="bf16", name=case, **STRESS[case])
        want = oracle_out(wl)
    g = gpu_out(B, wl, latency_mode=1)
    base = gpu_out(B, wl)
    assert np.isfinite(g).all()
    err = score_err(g, want)
    print(f"{case} {kind}: latency mode score error {err:.3e}; against the throughput configuration {score_err(g, base):.3e}")
    assert err <= TOL_HOT["bf16"], err
    assert score_err(g, base) <= TOL_HOT["bf16"]


def test_latency_mode_determinism_and_independence(B):
    wl = stress(dtype="bf16", name="S4", hot=True, **STRESS["S4"])
    a = gpu_out(B, wl, latency_mode=1)
    assert np.array_equal(a, gpu_out(B, wl, latency_mode=1))
    co = wl.cand_offsets
    for i in range(wl.n_requests):
        assert np.array_equal(gpu_out(B, wl.subset([i]), latency_mode=1), a[co[i]:co[i + 1]])


@pytest.mark.parametrize("name", ["uniform", "jagged", "long"])
def test_latency_mode_on_benchmark_workloads(B, name):
    wl = W.make_workload(name)
    g = gpu_out(B, wl, latency_mode=1)
    co = wl.cand_offsets
    worst = 0.0
    for i in sample_requests(wl, name):
        worst = max(worst, score_err(g[co[i]:co[i + 1]], request_scores(wl, i)))
    print(f"{name}, latency mode: max score error {worst:.3e}")
    assert worst <= TOL["bf16"]


def test_latency_mode_is_ignored_by_fp32_handles(B):
    wl = stress(dtype="f32", name="S2", hot=True, **STRESS["S2"])
    assert np.array_equal(gpu_out(B, wl, latency_mode=1), gpu_out(B, wl))
    cfg = B.config_for(wl)
    cfg.latency_mode = 2
    with pytest.raises(B.FlameGRError) as e:
        B.flame_gr_create(cfg)
    assert e.value.code == -1


def test_latency_mode_graph_replay(B):
    """A handle in latency mode can be captured right after its creation (its kernels' launch attributes are set
    at create, not inside the capture) and replays what its eager forward computes."""
    import torch
    wl = stress(dtype="bf16", name="S6", hot=True, **STRESS["S6"])
    want = gpu_out(B, wl, latency_mode=1)
    h = B.flame_gr_create(B.config_for(wl, latency_mode=1))
    try:
        dw, hist, cand = B.to_device(wl)
        out = torch.zeros(int(wl.cand_offsets[-1]), device="cuda:0")
        B.flame_gr_capture(h, dw, hist, wl.history_offsets, cand, wl.cand_offsets, out)
        for _ in range(2):
            out.zero_()
            B.flame_gr_replay(h)
            torch.cuda.synchronize()
            assert np.array_equal(out.cpu().numpy(), want)
    finally:
        B.flame_gr_destroy(h)
