"""GPU parity of the two-stage path (history prefill with per-layer K/V kept on the device, then candidate
scoring against it) with the one-pass forward and with the fp64 CPU oracle.

A history row never looks at a candidate, so splitting the pass changes no operand of any sum and no order of
summation: the two-stage scores must equal the one-pass scores bit for bit, whatever the reserved capacity,
the stream grouping or the number of score calls per prefill.
"""
import numpy as np
import pytest

from paper_2509_22681_amd import workloads as W
from tests.test_gpu_parity import STRESS, TOL_HOT, oracle_all, run_gpu, score_err, stress

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2509_22681_amd import binding
    return binding


def two_stage(B, wl, *, capacity=None, n_streams=0, score_calls=1, slack_tokens=None):
    """prefill once, then score the full candidate set `score_calls` times; returns the list of score arrays."""
    import torch
    cap = np.diff(wl.cand_offsets).astype(np.int32) if capacity is None else np.asarray(capacity, np.int32)
    extra = int(cap.sum() - wl.cand_offsets[-1]) if slack_tokens is None else slack_tokens
    h = B.flame_gr_create(B.config_for(wl, n_streams=n_streams, kv_cache=1, slack_tokens=extra))
    try:
        dw, hist, cand = B.to_device(wl)
        B.flame_gr_prefill(h, dw, hist, wl.history_offsets, cap)
        outs = []
        for _ in range(score_calls):
            scores = torch.full((int(wl.cand_offsets[-1]),), float("nan"), device="cuda:0", dtype=torch.float32)
            B.flame_gr_score(h, dw, cand, wl.cand_offsets, scores)
            torch.cuda.synchronize()
            outs.append(scores.cpu().numpy().copy())
        return outs
    finally:
        B.flame_gr_destroy(h)


@pytest.mark.parametrize("case", ["S2", "S4", "S5", "S6"])
def test_two_stage_equals_one_pass_bit_for_bit(B, case):
    wl = stress(dtype="bf16", name=case, hot=True, **STRESS[case])
    ref, _ = run_gpu(B, wl)
    a, b = two_stage(B, wl, score_calls=2)
    assert np.array_equal(a, ref) and np.array_equal(b, ref)
    err = score_err(a, oracle_all(wl))
    print(f"{case}: two-stage score error against the oracle {err:.3e}")
    assert err <= TOL_HOT["bf16"], err


def test_reserved_capacity_and_stream_groups_change_nothing(B):
    wl = stress(dtype="bf16", name="S4", hot=True, **STRESS["S4"])
    ref, _ = run_gpu(B, wl)
    M = np.diff(wl.cand_offsets)
    for cap, ns in ((M + 1, 0), (M + 64, 3), (np.full_like(M, 300), 2), (M * 2 + 7, 5)):
        (g,) = two_stage(B, wl, capacity=cap, n_streams=ns)
        assert np.array_equal(g, ref), (cap, ns)


def test_candidate_micro_batches_against_one_prefill(B):
    """One prefill, then several score calls with different candidate subsets (also none for some request).
    A regrouped candidate may share its 32-row patch with other neighbours, and the attention kernel picks
    its SiLU route (polynomial or exact) per patch: regrouped scores agree to the polynomial's accuracy, the
    full set in the original order bit for bit."""
    import torch
    wl = stress([150, 64, 0, 300], [70, 128, 9, 40], 128, 2, "bf16", nb=16, D=256, name="micro")
    ref, _ = run_gpu(B, wl)
    co = wl.cand_offsets
    M = np.diff(co)
    h = B.flame_gr_create(B.config_for(wl, kv_cache=1))
    try:
        dw, hist, cand = B.to_device(wl)
        B.flame_gr_prefill(h, dw, hist, wl.history_offsets, M)
        rng = np.random.default_rng(11)
        for take in ([70, 128, 9, 40], [1, 0, 9, 13], [0, 0, 0, 0], [64, 65, 0, 40], [33, 128, 1, 0]):
            full = list(take) == list(M)
            idx = [co[i] + (np.arange(M[i]) if full else rng.permutation(M[i]))[:t] for i, t in enumerate(take)]
            flat = np.concatenate(idx).astype(np.int64)
            sub_off = np.concatenate([[0], np.cumsum(take)]).astype(np.int32)
            sub = cand[torch.from_numpy(flat).to("cuda:0")] if len(flat) else None
            out = torch.full((max(len(flat), 1),), float("nan"), device="cuda:0", dtype=torch.float32)
            B.flame_gr_score(h, dw, sub, sub_off, out if len(flat) else None)
            torch.cuda.synchronize()
            got = out.cpu().numpy()[:len(flat)]
            if full:
                assert np.array_equal(got, ref[flat])
            else:
                assert score_err(got, ref[flat]) <= 2e-3, (take, score_err(got, ref[flat]))
    finally:
        B.flame_gr_destroy(h)


@pytest.mark.parametrize("name", ["jagged", "long"])
def test_two_stage_on_benchmark_workloads(B, name):
    wl = W.make_workload(name)
    ref, _ = run_gpu(B, wl)
    (g,) = two_stage(B, wl)
    assert np.isfinite(g).all()
    assert np.array_equal(g, ref)


def test_two_stage_error_paths(B):
    import torch
    wl = stress([40, 10], [8, 20], 64, 2, "bf16", nb=16, D=128, name="errs")
    ref, _ = run_gpu(B, wl)
    dw, hist, cand = B.to_device(wl)
    scores = torch.zeros(28, device="cuda:0")
    M = np.diff(wl.cand_offsets)
    # a handle without the cache
    h = B.flame_gr_create(B.config_for(wl))
    try:
        with pytest.raises(B.FlameGRError) as e:
            B.flame_gr_prefill(h, dw, hist, wl.history_offsets, M)
        assert e.value.code == -5
        with pytest.raises(B.FlameGRError) as e:
            B.flame_gr_score(h, dw, cand, wl.cand_offsets, scores)
        assert e.value.code == -5
    finally:
        B.flame_gr_destroy(h)
    # the fp32 path has no two-stage kernels
    wf = stress([40], [8], 64, 2, "f32", nb=16, D=128, name="errs32")
    with pytest.raises(B.FlameGRError) as e:
        B.flame_gr_create(B.config_for(wf, kv_cache=1))
    assert e.value.code == -5
    h = B.flame_gr_create(B.config_for(wl, kv_cache=1, max_seq_tokens=0))
    try:
        with pytest.raises(B.FlameGRError) as e:                      # nothing cached yet
            B.flame_gr_score(h, dw, cand, wl.cand_offsets, scores)
        assert e.value.code == -1
        with pytest.raises(B.FlameGRError) as e:                      # capacity beyond the workspace
            B.flame_gr_prefill(h, dw, hist, wl.history_offsets, np.array([8, 5000], np.int32))
        assert e.value.code == -2
        with pytest.raises(B.FlameGRError) as e:
            B.flame_gr_prefill(h, dw, hist, wl.history_offsets, np.array([8, -1], np.int32))
        assert e.value.code == -1
        B.flame_gr_prefill(h, dw, hist, wl.history_offsets, M)
        with pytest.raises(B.FlameGRError) as e:                      # more candidates than reserved
            B.flame_gr_score(h, dw, cand, np.array([0, 9, 28], np.int32), scores)
        assert e.value.code == -2
        with pytest.raises(B.FlameGRError) as e:                      # another number of requests
            B.flame_gr_score(h, dw, cand, np.array([0, 8], np.int32), scores)
        assert e.value.code == -1
        with pytest.raises(B.FlameGRError) as e:
            B.flame_gr_score(h, dw, None, wl.cand_offsets, scores)
        assert e.value.code == -1
        # the cache survives the rejected calls
        scores.fill_(float("nan"))
        B.flame_gr_score(h, dw, cand, wl.cand_offsets, scores)
        torch.cuda.synchronize()
        assert np.array_equal(scores.cpu().numpy(), ref)
        # a one-pass forward on the handle has its own planes: the cache stays valid
        scores.fill_(float("nan"))
        B.flame_gr_forward(h, dw, hist, wl.history_offsets, cand, wl.cand_offsets, scores)
        torch.cuda.synchronize()
        assert np.array_equal(scores.cpu().numpy(), ref)
        scores.fill_(float("nan"))
        B.flame_gr_score(h, dw, cand, wl.cand_offsets, scores)
        torch.cuda.synchronize()
        assert np.array_equal(scores.cpu().numpy(), ref)
        # and an empty prefill followed by an empty score is legal
        B.flame_gr_prefill(h, dw, None, np.zeros(1, np.int32), np.zeros(0, np.int32))
        B.flame_gr_score(h, dw, None, np.zeros(1, np.int32), None)
        torch.cuda.synchronize()
    finally:
        B.flame_gr_destroy(h)
