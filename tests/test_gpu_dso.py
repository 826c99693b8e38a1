"""GPU tests of the explicit-shape executors: the forward captured as a HIP graph (flame_gr_capture / flame_gr_replay)
and the request orchestrator built from such executors (flame_dso_*), against the eager forward and the fp64 oracle.
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


# ------------------------------------------------------------------ graph capture and replay
@pytest.mark.parametrize("dtype,case", [("bf16", "S4"), ("bf16", "S5"), ("f32", "S2")])
def test_replay_matches_eager_on_every_replay(B, dtype, case):
    """The graph is replayed several times, with new input contents written in place, eager work of the same
    process and synchronisations in between, and every replay is checked against the eager forward."""
    import torch
    wl = stress(dtype=dtype, name=case, hot=True, **STRESS[case])
    dw, hist, cand = B.to_device(wl)
    n = int(wl.cand_offsets[-1])
    h_graph = B.flame_gr_create(B.config_for(wl))
    h_eager = B.flame_gr_create(B.config_for(wl))
    try:
        got = torch.full((n,), float("nan"), device="cuda:0")
        want = torch.full((n,), float("nan"), device="cuda:0")
        B.flame_gr_capture(h_graph, dw, hist, wl.history_offsets, cand, wl.cand_offsets, got)
        assert torch.isnan(got).all().item()              # capturing runs nothing
        side = torch.cuda.Stream()
        gen = torch.Generator(device="cuda:0").manual_seed(5)
        for it in range(5):
            if it:                                        # new request contents, same shape, same buffers
                hist.copy_(torch.randn(hist.shape, device="cuda:0", generator=gen).to(hist.dtype))
                cand.copy_(torch.randn(cand.shape, device="cuda:0", generator=gen).to(cand.dtype))
            got.fill_(float("nan"))
            torch.cuda.synchronize()
            B.flame_gr_replay(h_graph, stream=side if it % 2 else None)
            B.flame_gr_forward(h_eager, dw, hist, wl.history_offsets, cand, wl.cand_offsets, want)
            torch.cuda.synchronize()
            assert torch.equal(got, want), f"replay {it}"
            (torch.ones(1 << 16, device="cuda:0") * 3).sum().item()      # unrelated eager work between replays
    finally:
        B.flame_gr_destroy(h_graph)
        B.flame_gr_destroy(h_eager)


def test_first_replay_against_the_oracle(B):
    import torch
    wl = stress(dtype="bf16", name="S6", hot=True, **STRESS["S6"])
    dw, hist, cand = B.to_device(wl)
    h = B.flame_gr_create(B.config_for(wl))
    try:
        got = torch.zeros(int(wl.cand_offsets[-1]), device="cuda:0")
        B.flame_gr_capture(h, dw, hist, wl.history_offsets, cand, wl.cand_offsets, got)
        B.flame_gr_replay(h)
        torch.cuda.synchronize()
        err = score_err(got.cpu().numpy(), oracle_all(wl))
        print(f"graph replay: score error against the oracle {err:.3e}")
        assert err <= TOL_HOT["bf16"]
    finally:
        B.flame_gr_destroy(h)


def test_capture_error_paths_and_invalidation(B):
    import torch
    wl = stress([40, 10], [8, 20], 64, 2, "bf16", nb=16, D=128, name="cap")
    ref, _ = run_gpu(B, wl)
    dw, hist, cand = B.to_device(wl)
    scores = torch.zeros(28, device="cuda:0")
    h = B.flame_gr_create(B.config_for(wl, n_streams=2))
    try:
        with pytest.raises(B.FlameGRError) as e:              # stream groups are not captured
            B.flame_gr_capture(h, dw, hist, wl.history_offsets, cand, wl.cand_offsets, scores)
        assert e.value.code == -5
    finally:
        B.flame_gr_destroy(h)
    h = B.flame_gr_create(B.config_for(wl))
    try:
        with pytest.raises(B.FlameGRError) as e:              # nothing captured yet
            B.flame_gr_replay(h)
        assert e.value.code == -1
        with pytest.raises(B.FlameGRError) as e:              # no candidates: nothing to capture
            B.flame_gr_capture(h, dw, hist, wl.history_offsets, None, np.zeros(3, np.int32), None)
        assert e.value.code == -1
        with pytest.raises(B.FlameGRError) as e:              # bad offsets are rejected before any capture starts
            B.flame_gr_capture(h, dw, hist, np.array([0, 50, 40], np.int32), cand, wl.cand_offsets, scores)
        assert e.value.code == -1
        B.flame_gr_capture(h, dw, hist, wl.history_offsets, cand, wl.cand_offsets, scores)
        B.flame_gr_replay(h)
        torch.cuda.synchronize()
        assert np.array_equal(scores.cpu().numpy(), ref)
        # capturing again replaces the graph (another shape: the first request alone)
        one = torch.zeros(8, device="cuda:0")
        B.flame_gr_capture(h, dw, hist, wl.history_offsets[:2], cand, wl.cand_offsets[:2], one)
        B.flame_gr_replay(h)
        torch.cuda.synchronize()
        assert np.array_equal(one.cpu().numpy(), ref[:8])
        # a second slot holds another shape side by side; eager forwards in between stage their own plan
        # tables and leave both graphs intact
        B.flame_gr_capture(h, dw, hist, wl.history_offsets, cand, wl.cand_offsets, scores, slot=3)
        for _ in range(2):
            scores.fill_(float("nan"))
            B.flame_gr_forward(h, dw, hist, wl.history_offsets, cand, wl.cand_offsets, scores)
            torch.cuda.synchronize()
            assert np.array_equal(scores.cpu().numpy(), ref)
            one.fill_(float("nan"))
            B.flame_gr_replay(h, slot=0)
            torch.cuda.synchronize()
            assert np.array_equal(one.cpu().numpy(), ref[:8])
            scores.fill_(float("nan"))
            B.flame_gr_replay(h, slot=3)
            torch.cuda.synchronize()
            assert np.array_equal(scores.cpu().numpy(), ref)
        for slot in (1, -1, 16):
            with pytest.raises(B.FlameGRError) as e:          # empty slot, slots out of range
                B.flame_gr_replay(h, slot=slot)
            assert e.value.code == -1
        with pytest.raises(B.FlameGRError) as e:
            B.flame_gr_capture(h, dw, hist, wl.history_offsets, cand, wl.cand_offsets, scores, slot=16)
        assert e.value.code == -1
    finally:
        B.flame_gr_destroy(h)


# ------------------------------------------------------------------ orchestrator
def _requests(wl_cfg, L, Ms, seed, dtype):
    """One user per request: one set of model weights, own history and candidates per request."""
    base = W.make_custom([L], [1], d=wl_cfg["d"], H=wl_cfg["H"], n_layers=wl_cfg["layers"], n_buckets=16, max_rel_dist=256,
                         dtype=dtype, seed=seed, emb_std=1.0, rab_std=1.0, bias_amp=0.1, affine_random=True, name="base")
    out = []
    for k, M in enumerate(Ms):
        rng = np.random.default_rng(1000 + k)
        h = W._round_storage(rng.standard_normal((L, wl_cfg["d"])).astype(np.float32), dtype)
        c = W._round_storage(rng.standard_normal((M, wl_cfg["d"])).astype(np.float32), dtype)
        out.append(W.Workload(f"req{k}", base.cfg, np.array([0, L], np.int32), np.array([0, M], np.int32), h, c, base.weights))
    return out


@pytest.mark.parametrize("dtype,explicit", [("bf16", True), ("bf16", False), ("f32", True), ("bf16", 2), ("f32", 2)])
def test_orchestrator_scores_every_request(B, dtype, explicit):
    import torch
    shape = dict(d=64, H=2, layers=2)
    L, profiles = 100, [16, 32, 64]
    Ms = [16, 32, 64, 1, 17, 40, 64, 150, 33, 16, 200, 5]
    reqs = _requests(shape, L, Ms, seed=21, dtype=dtype)
    dw, _, _ = B.to_device(reqs[0])
    cfg = B.config_for(reqs[0])
    dso = B.flame_dso_create(cfg, dw, L, profiles, n_executors=3, explicit_shapes=explicit, max_batch=3)
    try:
        outs = [np.full(M, np.nan, np.float32) for M in Ms]
        tickets = []
        for r, o in zip(reqs, outs):
            tickets.append(B.flame_dso_submit(dso, B.host_embedding(r.history_emb, dtype), B.host_embedding(r.cand_emb, dtype), o))
        for t in reversed(tickets):                       # any order; retired tickets return at once
            B.flame_dso_wait(dso, t)
        B.flame_dso_wait(dso, tickets[0])
        st = B.flame_dso_stats(dso)
        assert st["requests"] == len(Ms)
        if explicit == 2:       # micro-batches of up to 3 requests: fewer forwards than requests, no padded rows
            assert st["chunks"] < len(Ms) and st["candidate_rows_computed"] == sum(Ms)
        else:
            assert st["chunks"] >= len(Ms) and st["waits_for_a_busy_executor"] > 0
        worst = 0.0
        for r, o in zip(reqs, outs):
            assert np.isfinite(o).all()
            worst = max(worst, score_err(o, oracle_all(r)))
        print(f"orchestrator ({dtype}, explicit={explicit}): max score error against the oracle {worst:.3e}")
        assert worst <= TOL_HOT[dtype]
        # a request served in one exact chunk equals the eager forward of that request bit for bit
        for k in (0, 1, 2):
            eager, _ = run_gpu(B, reqs[k])
            if dtype == "f32" and explicit == 2:      # fp32 kernels: equal up to the order of a few sums
                assert np.allclose(outs[k], eager, rtol=1e-5, atol=1e-6)
            else:
                assert np.array_equal(outs[k], eager)
        with pytest.raises(B.FlameGRError) as e:
            B.flame_dso_wait(dso, 10 ** 6)
        assert e.value.code == -1
        with pytest.raises(B.FlameGRError) as e:
            B.flame_dso_submit(dso, B.host_embedding(reqs[0].history_emb, dtype), np.zeros((0, 64), np.uint16), np.zeros(0, np.float32))
        assert e.value.code == -1
        # still serving after the rejected calls, and a drain delivers everything outstanding
        again = np.full(Ms[4], np.nan, np.float32)
        B.flame_dso_submit(dso, B.host_embedding(reqs[4].history_emb, dtype), B.host_embedding(reqs[4].cand_emb, dtype), again)
        if explicit == 2:
            B.flame_dso_flush(dso)
        B.flame_dso_drain(dso)
        assert np.allclose(again, outs[4], rtol=1e-5, atol=1e-6) if dtype == "f32" else np.array_equal(again, outs[4])
    finally:
        B.flame_dso_destroy(dso)


def test_orchestrator_rejects_bad_configurations(B):
    wl = stress([10], [4], 64, 2, "bf16", nb=16, D=128, name="dsoerr")
    dw, _, _ = B.to_device(wl)
    cfg = B.config_for(wl)
    for kw in (dict(profiles=[], n_executors=1), dict(profiles=[8, 4], n_executors=1),
               dict(profiles=[4], n_executors=0), dict(profiles=[4], n_executors=257),
               dict(profiles=[4], n_executors=1, explicit_shapes=3), dict(profiles=[4], n_executors=1, explicit_shapes=2, max_batch=0)):
        with pytest.raises(B.FlameGRError) as e:
            B.flame_dso_create(cfg, dw, 10, **kw)
        assert e.value.code == -1
    bad = B.config_for(wl)
    bad.n_heads = 5                                        # d_model not a multiple of n_heads
    with pytest.raises(B.FlameGRError) as e:
        B.flame_dso_create(bad, dw, 10, [4], 1)
    assert e.value.code == -1


def test_micro_batches_of_mixed_history_lengths(B):
    """Mode 2 with flame_dso_submit_jagged: requests of different history and candidate lengths share micro-batches;
    every request's scores equal those of its own eager forward (a request never sees its batch)."""
    wl = stress([200, 10, 64, 333, 0, 129], [40, 300, 1, 17, 5, 64], 64, 2, "bf16", nb=16, D=512, name="mixed")
    dw, _, _ = B.to_device(wl)
    ref, _ = run_gpu(B, wl)
    ho, co = wl.history_offsets, wl.cand_offsets
    dso = B.flame_dso_create(B.config_for(wl), dw, 400, [128, 300], n_executors=2, explicit_shapes=2, max_batch=4)
    try:
        outs = [np.full(int(co[i + 1] - co[i]), np.nan, np.float32) for i in range(wl.n_requests)]
        tickets = [B.flame_dso_submit_jagged(dso, B.host_embedding(wl.history_emb[ho[i]:ho[i + 1]], "bf16"),
                                             B.host_embedding(wl.cand_emb[co[i]:co[i + 1]], "bf16"), outs[i])
                   for i in range(wl.n_requests)]
        for t in tickets:
            B.flame_dso_wait(dso, t)
        for i in range(wl.n_requests):
            assert np.array_equal(outs[i], ref[co[i]:co[i + 1]]), i
        with pytest.raises(B.FlameGRError) as e:                      # a history beyond the capacity
            B.flame_dso_submit_jagged(dso, np.zeros((401, 64), np.uint16), np.zeros((1, 64), np.uint16), np.zeros(1, np.float32))
        assert e.value.code == -2
    finally:
        B.flame_dso_destroy(dso)
    dso = B.flame_dso_create(B.config_for(wl), dw, 400, [128, 300], n_executors=1, explicit_shapes=0)
    try:
        with pytest.raises(B.FlameGRError) as e:                      # only the micro-batch mode takes other lengths
            B.flame_dso_submit_jagged(dso, np.zeros((10, 64), np.uint16), np.zeros((1, 64), np.uint16), np.zeros(1, np.float32))
        assert e.value.code == -5
    finally:
        B.flame_dso_destroy(dso)
