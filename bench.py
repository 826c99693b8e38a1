#!/usr/bin/env python3
"""Throughput benchmark of the GR forward on one MI355X.

A step is one flame_gr_forward over the whole synthetic batch (all kernels of the hot path).
Inputs are resident in HBM before the timed region.  Prints ONE JSON line:
candidate scores/s, ms per step, the roofline of the dominant kernel (attention, bf16 MFMA) from
HIP-event timings taken on the launch stream inside the timed region, and the CPU oracle timed on
a bounded sample of the same workload on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense MFMA peak, the same for bf16 and fp16 operands


def attention_flops_per_layer(cfg, L, M):
    """(full layer, last layer) algorithmic attention flops: 4*d per allowed (query, key) pair."""
    L = L.astype(np.float64)
    M = M.astype(np.float64)
    full = 4.0 * cfg.d_model * (L * (L + 1) / 2 + M * (L + 1)).sum()
    last = 4.0 * cfg.d_model * (M * (L + 1)).sum()
    return full, last


def source_digest(*names):
    """sha256 over the named kernel sources: what a stored counter measurement is tied to."""
    import hashlib
    h = hashlib.sha256()
    for n in names:
        with open(os.path.join(ROOT, "paper_2509_22681_amd", "csrc", n), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


ATTN_SOURCES = ("attn_mfma.hip", "device_common.h", "plan.cpp")


def stored_traffic(workload, launches_per_step):
    """HBM bytes per attention launch from the committed rocprofv3 --pmc summary of this workload (two counter
    runs, FETCH_SIZE and WRITE_SIZE, scaled by a copy kernel of known size).  A stored measurement: counters cannot
    be read from inside this process.  It is tied to the kernel it was taken on: if the attention kernel's sources
    or the number of attention launches per forward differ from what the summary records, it is stale and not reported."""
    path = os.path.join(ROOT, "profiles", f"{workload}_attn_hbm_traffic.json")
    try:
        with open(path) as f:
            rec = json.load(f)
        if rec.get("kernel_sources_sha256_16") != source_digest(*ATTN_SOURCES):
            return None, "stored measurement is of another version of the attention kernel (source digest differs)"
        if int(rec.get("attention_launches_per_forward", -1)) != int(launches_per_step):
            return None, "stored measurement is of another launch sequence"
        return float(rec["bytes_per_launch"]), None
    except (OSError, KeyError, ValueError):
        return None, "no stored measurement for this workload"


def measured_mfma_peak_tflops():
    """The matrix-instruction rate this chip sustains on random data fed from LDS (profiles/chip_microbench.json, the
    output of paper_2509_22681_amd/chip_microbench): the clock drops under matrix load, so the published peak is
    not reachable with real operands."""
    try:
        with open(os.path.join(ROOT, "profiles", "chip_microbench.json")) as f:
            return float(json.load(f)["mfma_f16_random_data_lds_fed_tflops"])
    except (OSError, KeyError, ValueError):
        return None


def cpu_baseline(wl, budget_s=25.0):
    """Time the fp64 oracle, as it stands, on a stratified sample of the workload's requests: the cheapest, the median
    and the most expensive by the cost model plus two seeded picks, taken cheapest first until the time budget is
    used (at least two).  The whole batch is extrapolated with a two-term model fitted to the timed requests,
    t = a * projection flops + b * N^2 * heads * layers (the oracle evaluates the full N x N score matrix per head with
    elementwise numpy, which does not scale like the flops), falling back to flops alone with fewer than two samples."""
    import oracle
    L, M = wl.L.astype(np.float64), wl.M.astype(np.float64)
    c = wl.cfg
    N = L + M
    gemm = c.n_layers * 10.0 * N * c.d_model ** 2
    elem = c.n_layers * c.n_heads * N * N
    cost = gemm + 4.0 * c.d_model * c.n_layers * N * N
    order = np.argsort(cost, kind="stable")
    picks = [int(order[0]), int(order[len(order) // 2]), int(order[-1])]
    for r in np.random.default_rng(2024).permutation(wl.n_requests):
        if len(picks) >= min(5, wl.n_requests):
            break
        if int(r) not in picks:
            picks.append(int(r))
    picks = sorted(set(picks), key=lambda i: cost[i])
    cfgd = c.to_dict()
    ho, co = wl.history_offsets, wl.cand_offsets
    t0 = time.perf_counter()
    done, times = [], []
    for i in picks:
        if len(done) >= 2 and time.perf_counter() - t0 > budget_s:
            break
        if len(done) >= 1:
            # do not start a request that would carry the sample well past the budget
            est = times[-1] * cost[i] / cost[done[-1]]
            if len(done) >= 2 and time.perf_counter() - t0 + est > 1.2 * budget_s:
                break
        t1 = time.perf_counter()
        oracle.forward_request(cfgd, wl.weights, wl.history_emb[ho[i]:ho[i + 1]], wl.cand_emb[co[i]:co[i + 1]])
        times.append(time.perf_counter() - t1)
        done.append(i)
    dt = time.perf_counter() - t0
    times = np.array(times)
    if len(done) >= 2:
        A = np.stack([gemm[done], elem[done]], 1)
        coef, _ = __import__("scipy.optimize", fromlist=["nnls"]).nnls(A / times[:, None], np.ones(len(done)))
        est_total_s = float(coef[0] * gemm.sum() + coef[1] * elem.sum())
        model = "t = a * projection flops + b * N^2 * heads * layers, non-negative least squares on the timed requests"
    else:
        est_total_s = float(times.sum() * cost.sum() / cost[done].sum())
        model = "flops"
    nsc = int(M[done].sum())
    return {
        "value": float(M.sum()) / est_total_s, "unit": "candidate scores/s", "cores": len(os.sched_getaffinity(0)),
        "kind": "oracle",
        "sample": f"{len(done)} of {wl.n_requests} requests, stratified by cost (cheapest, median, most expensive, two seeded "
                  f"picks; cheapest first within the time budget): requests {done} with (L, M) = "
                  f"{[(int(L[i]), int(M[i])) for i in done]}, {nsc} scores in {dt:.1f} s; whole batch extrapolated to "
                  f"{est_total_s:.0f} s ({model})",
        "seconds_per_timed_request": [float(t) for t in times],
    }


def small_workloads_leg(B, steps=50):
    """The two small workloads of the benchmark definition (one tiny fp32 request; 32 uniform requests), which are
    bound by launches rather than by arithmetic: eager forwards against replays of the forward captured as a HIP graph
    (the explicit-shape executor of Section 3.3), both with weights declared static."""
    import torch
    from paper_2509_22681_amd import workloads as W
    out = {}
    for name in ("tiny_f32", "uniform"):
        wl = W.make_workload(name)
        dw, hist, cand = B.to_device(wl)
        ws = B.pack_weights(dw)
        scores = torch.zeros(int(wl.cand_offsets[-1]), device="cuda:0", dtype=torch.float32)
        res = {}
        for static in (0, 1):
            h = B.flame_gr_create(B.config_for(wl, weights_static=static))
            try:
                for _ in range(5):
                    B.flame_gr_forward(h, ws, hist, wl.history_offsets, cand, wl.cand_offsets, scores)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(steps):
                    B.flame_gr_forward(h, ws, hist, wl.history_offsets, cand, wl.cand_offsets, scores)
                torch.cuda.synchronize()
                res["eager_ms_per_forward" + ("_weights_static" if static else "")] = (time.perf_counter() - t0) / steps * 1e3
                if static:
                    eager = scores.clone()
                    s = torch.cuda.Stream()
                    B.flame_gr_capture(h, ws, hist, wl.history_offsets, cand, wl.cand_offsets, scores, record_stream=s)
                    for _ in range(5):
                        B.flame_gr_replay(h, stream=s)
                    s.synchronize()
                    t0 = time.perf_counter()
                    for _ in range(steps):
                        B.flame_gr_replay(h, stream=s)
                    s.synchronize()
                    ms = (time.perf_counter() - t0) / steps * 1e3
                    res["graph_replay_ms_per_forward"] = ms
                    res["graph_replay_scores_per_s"] = scores.numel() / (ms * 1e-3)
                    res["replay_equals_eager"] = bool(torch.equal(scores, eager))
            finally:
                torch.cuda.synchronize()
                B.flame_gr_destroy(h)
        out[name] = res
    return out


def request_mode_latency(B, wl, dw, hist, cand, concurrency=1, max_requests=128, latency_mode=0):
    """Requests submitted one per call in a closed loop over `concurrency` executors (handles), each with its
    own stream (the executor pool of Section 3.3): per-request latency from submission to scores ready
    (HIP events on the executor's stream, recorded right before the call and right after its last kernel),
    and the throughput of that mode."""
    import torch
    Bn = wl.n_requests
    idx = list(range(Bn)) if Bn <= max_requests else list(np.linspace(0, Bn - 1, max_requests).astype(int))
    L, M = wl.L, wl.M
    c = wl.cfg
    cfg = B.make_config(c.n_layers, c.d_model, c.n_heads, c.n_buckets, c.max_rel_dist, c.dtype, ln_eps=c.ln_eps,
                        attn_scale=c.attn_scale, max_requests=1, max_total_tokens=int((L + M).max()),
                        latency_mode=latency_mode, weights_static=1)      # serving: the weights are frozen (Section 3.3)
    ws = B.pack_weights(dw)
    ho, co = wl.history_offsets, wl.cand_offsets
    E = max(1, concurrency)
    handles = [B.flame_gr_create(cfg) for _ in range(E)]
    streams = [torch.cuda.Stream() for _ in range(E)]
    scores = [torch.zeros(int(M.max()), device="cuda:0", dtype=torch.float32) for _ in range(E)]
    pending = [None] * E            # (start event, end event) of the request in flight on executor e
    lat = []
    try:
        for rep in range(2):           # first pass warms up
            lat = []
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for n, i in enumerate(idx):
                e = n % E
                if pending[e] is not None:          # the executor is free once its previous request is done
                    pending[e][1].synchronize()
                    lat.append(pending[e][0].elapsed_time(pending[e][1]))
                hh, cc = hist[ho[i]:ho[i + 1]], cand[co[i]:co[i + 1]]
                o1 = np.array([0, L[i]], np.int32)
                o2 = np.array([0, M[i]], np.int32)
                ev0 = torch.cuda.Event(enable_timing=True)
                ev1 = torch.cuda.Event(enable_timing=True)
                ev0.record(streams[e])
                B.flame_gr_forward(handles[e], ws, hh, o1, cc, o2, scores[e], stream=streams[e])
                ev1.record(streams[e])
                pending[e] = (ev0, ev1)
            for e in range(E):
                if pending[e] is not None:
                    pending[e][1].synchronize()
                    lat.append(pending[e][0].elapsed_time(pending[e][1]))
                    pending[e] = None
            wall = time.perf_counter() - t0
    finally:
        torch.cuda.synchronize()
        for h in handles:
            B.flame_gr_destroy(h)
    lat = np.array(lat)
    return {"concurrency": E, "attention_latency_configuration": bool(latency_mode), "weights_static": True, "p50_ms": float(np.percentile(lat, 50)), "p99_ms": float(np.percentile(lat, 99)),
            "mean_ms": float(lat.mean()), "requests": len(idx),
            "scores_per_s": float(M[idx].sum() / wall)}


def mixed_traffic_leg(B, wl, dw, n_requests=320, n_executors=4, hist_len=1024,
                      profiles=(128, 256, 512, 1024), seed=0):
    """The paper's mixed-traffic experiment (Section 4.2.3, DSO table) on this model: single-user requests with a
    history of 1024 items and a candidate count drawn uniformly from {128, 256, 512, 1024}, host embeddings in,
    host scores out, served in a closed loop by the orchestrator: once with explicit-shape executors (one captured
    graph per profile on every executor), once with the implicit-shape baseline (same pool, dynamic-shape eager
    forward), and with jagged micro-batches (2 executors that gather 4 or 8 requests per jagged forward).
    Latency is host wall-clock from submit to scores delivered."""
    c = wl.cfg
    cfg = B.make_config(c.n_layers, c.d_model, c.n_heads, c.n_buckets, c.max_rel_dist, c.dtype, ln_eps=c.ln_eps,
                        attn_scale=c.attn_scale)
    rng = np.random.default_rng(seed)
    Ms = rng.choice(np.asarray(profiles), size=n_requests)
    pool = 8                                   # distinct users; every request gets its own candidate slice
    std = 0.1
    from paper_2509_22681_amd import workloads as W
    hist_pool = [B.host_embedding(W._round_storage(rng.standard_normal((hist_len, c.d_model)).astype(np.float32) * std, c.dtype), c.dtype)
                 for _ in range(pool)]
    cand_pool = B.host_embedding(W._round_storage(rng.standard_normal((max(profiles) * 2, c.d_model)).astype(np.float32) * std, c.dtype), c.dtype)
    out = {"hist_len": hist_len, "profiles": list(profiles), "requests": n_requests,
           "user_item_pairs": int(Ms.sum())}
    # executors = streams; how many of them run side by side depends on how the runtime maps the process's
    # streams onto its four hardware queues, so the per-request modes are run at two pool sizes
    modes = []
    for n_ex in sorted({3, n_executors}):
        modes += [(f"explicit_shape_{n_ex}_executors", 1, n_ex, 1, n_ex), (f"implicit_shape_{n_ex}_executors", 0, n_ex, 1, n_ex)]
    modes += [("jagged_micro_batch_4", 2, 2, 4, 8), ("jagged_micro_batch_8", 2, 2, 8, 16)]
    for mode, explicit, n_ex, max_batch, depth in modes:
        dso = B.flame_dso_create(cfg, dw, hist_len, list(profiles), n_ex, explicit_shapes=explicit, max_batch=max_batch)
        try:
            res = None
            for rep in range(2):               # first pass warms up
                lat, inflight = [], []
                outs = [np.empty(int(m), np.float32) for m in Ms]
                t0 = time.perf_counter()
                for k, m in enumerate(Ms):
                    if len(inflight) == depth:
                        t, ts = inflight.pop(0)
                        B.flame_dso_wait(dso, t)
                        lat.append(time.perf_counter() - ts)
                    off = int(rng.integers(0, max(profiles)))
                    ts = time.perf_counter()
                    t = B.flame_dso_submit(dso, hist_pool[k % pool], cand_pool[off:off + int(m)], outs[k])
                    inflight.append((t, ts))
                for t, ts in inflight:
                    B.flame_dso_wait(dso, t)
                    lat.append(time.perf_counter() - ts)
                wall = time.perf_counter() - t0
                assert all(np.isfinite(o).all() for o in outs), "non-finite scores"
                lat = np.array(lat) * 1e3
                res = {"user_item_pairs_per_s": float(Ms.sum() / wall), "mean_latency_ms": float(lat.mean()),
                       "p50_latency_ms": float(np.percentile(lat, 50)), "p99_latency_ms": float(np.percentile(lat, 99)),
                       "requests_per_s": float(n_requests / wall)}
            res.update(B.flame_dso_stats(dso))
            res.update({"executors": n_ex, "requests_in_flight": depth, "max_batch": max_batch})
            out[mode] = res
        finally:
            B.flame_dso_destroy(dso)
    return out


def climber_leg(B, steps=10, n_users=64, d=192, H=3, layers=12, n_blocks=2, E=256, T=2):
    """The paper's own model in the reading of include/flame_climber.h, at the two scenarios of its Table 2
    (base: sequence 512 + 128 candidates; long: 1024 + 512; 2 blocks x 12 layers): softmax attention with
    temperature, each block stack on its own handle, then gating fusion and task head.  d = 192 puts
    the block stacks' flops per request at 4.6e9 (base) and 1.63e10 (long) against the paper's 3.72e9 and 1.64e10.
    Reports batched throughput (n_users requests per pass), single-request latency, and the deviation of one
    request from the fp64 oracle."""
    import torch
    import oracle
    from paper_2509_22681_amd import workloads as W
    out = {"d_model": d, "n_heads": H, "layers_per_block": layers, "blocks": n_blocks, "expert_width": E, "tasks": T,
           "users_per_pass": n_users}
    rng = np.random.default_rng(0)
    head = dict(wg=(rng.standard_normal((n_blocks, d, n_blocks * d)) / np.sqrt(n_blocks * d)).astype(np.float32),
                cg=np.zeros((n_blocks, d), np.float32),
                a_w=(rng.standard_normal((T, E, d)) / np.sqrt(d)).astype(np.float32), a_b=np.zeros((T, E), np.float32),
                v=(rng.standard_normal((T, E)) / np.sqrt(E)).astype(np.float32), c=np.zeros(T, np.float32))
    head_dev = {k: torch.from_numpy(v).to("cuda:0") for k, v in head.items()}
    for name, L, M in (("base", 512, 128), ("long", 1024, 512)):
        wls = [W.make_custom([L] * n_users, [M] * n_users, d=d, H=H, n_layers=layers, n_buckets=128, max_rel_dist=1024,
                             dtype="bf16", seed=100 + b, attn_kind="softmax", name=f"{name}{b}") for b in range(n_blocks)]
        base = wls[0]
        res = {}
        for users in (n_users, 1):
            sub = base.subset(range(users))
            n = int(sub.cand_offsets[-1])
            handles, args, streams, hidden = [], [], [], []
            try:
                for b in range(n_blocks):
                    lo, hi = B.flame_climber_block_range(L, n_blocks, b)
                    hist = np.concatenate([sub.history_emb[i * L + lo:i * L + hi] for i in range(users)], 0)
                    ho = (np.arange(users + 1) * (hi - lo)).astype(np.int32)
                    wl_b = W.Workload(f"{name}{b}", base.cfg, ho, sub.cand_offsets, hist, sub.cand_emb, wls[b].weights)
                    handles.append(B.flame_gr_create(B.config_for(wl_b)))
                    dw, dh, dc = B.to_device(wl_b)
                    args.append((B.pack_weights(dw), dw, dh, ho, dc))
                    streams.append(torch.cuda.Stream())
                    hidden.append(torch.zeros((n, d), device="cuda:0", dtype=torch.float32))
                fused = torch.empty((n, d), device="cuda:0", dtype=torch.float32)
                probs = torch.zeros((n, T), device="cuda:0", dtype=torch.float32)
                main = torch.cuda.current_stream()

                # a pass of many users fills the chip block by block: one stream (two streams are faster only when the
                # runtime happens to put them on different hardware queues); a single request does not fill it, and
                # its block stacks run side by side on two streams
                side = users == 1

                def one_pass():
                    for b in range(n_blocks):
                        if side:
                            streams[b].wait_stream(main)
                        ws, _, dh, ho, dc = args[b]
                        B.flame_gr_forward_hidden(handles[b], ws, dh, ho, dc, sub.cand_offsets, hidden[b],
                                                  stream=streams[b] if side else main)
                    if side:
                        for b in range(n_blocks):
                            main.wait_stream(streams[b])
                    B.flame_climber_head(head_dev, hidden, fused, probs)

                for _ in range(3):
                    one_pass()
                torch.cuda.synchronize()
                if users > 1:
                    t0 = time.perf_counter()
                    for _ in range(steps):
                        one_pass()
                    torch.cuda.synchronize()
                    ms = (time.perf_counter() - t0) / steps * 1e3
                    res["ms_per_pass"] = ms
                    res["user_item_pairs_per_s"] = n / (ms * 1e-3)
                    got = probs[:M].cpu().numpy()
                    want = oracle.climber_request(base.cfg.to_dict(), [w.weights for w in wls], head,
                                                  base.history_emb[:L], base.cand_emb[:M])
                    res["max_abs_prob_error_vs_oracle_request0"] = float(np.abs(got - want).max())
                else:
                    lat = []
                    for _ in range(30):
                        t0 = time.perf_counter()
                        one_pass()
                        torch.cuda.synchronize()
                        lat.append((time.perf_counter() - t0) * 1e3)
                    res["single_request_latency_ms_p50"] = float(np.percentile(lat, 50))
                    res["single_request_latency_ms_p99"] = float(np.percentile(lat, 99))
            finally:
                torch.cuda.synchronize()
                for h in handles:
                    B.flame_gr_destroy(h)
        Nb, Pb = L // n_blocks + M, (L // n_blocks) * (L // n_blocks + 1) // 2 + M * (L // n_blocks + 1)
        res["block_stack_flops_per_request"] = float(n_blocks * layers * (10 * Nb * d * d + 4 * Pb * d))
        out[name] = res
    return out


def production_serving_leg(B, wl, dw, max_requests=256):
    """The benchmark workload's own requests (history and candidate lengths as drawn) served from host memory by
    the orchestrator's jagged micro-batch mode: embeddings copied into pinned buffers, uploaded, scored in jagged
    forwards of up to max_batch requests, scores downloaded.  The PCIe-inclusive counterpart of the headline."""
    c = wl.cfg
    cfg = B.make_config(c.n_layers, c.d_model, c.n_heads, c.n_buckets, c.max_rel_dist, c.dtype, ln_eps=c.ln_eps,
                        attn_scale=c.attn_scale)
    ho, co = wl.history_offsets, wl.cand_offsets
    idx = [i % wl.n_requests for i in range(max_requests)]
    hist = [B.host_embedding(wl.history_emb[ho[i]:ho[i + 1]], c.dtype) for i in range(wl.n_requests)]
    cand = [B.host_embedding(wl.cand_emb[co[i]:co[i + 1]], c.dtype) for i in range(wl.n_requests)]
    n_scores = int(sum(len(cand[i]) for i in idx))
    out = {"requests": len(idx), "scores": n_scores,
           "host_bytes_per_request_mean": float(np.mean([hist[i].nbytes + cand[i].nbytes for i in idx]))}
    for max_batch, depth in ((4, 8), (8, 16)):
        dso = B.flame_dso_create(cfg, dw, int(wl.L.max()), [int(wl.M.max())], 2, explicit_shapes=2, max_batch=max_batch)
        try:
            res = None
            for rep in range(2):               # first pass warms up
                lat, inflight = [], []
                outs = [np.empty(len(cand[i]), np.float32) for i in idx]
                t0 = time.perf_counter()
                for k, i in enumerate(idx):
                    if len(inflight) == depth:
                        t, ts = inflight.pop(0)
                        B.flame_dso_wait(dso, t)
                        lat.append(time.perf_counter() - ts)
                    ts = time.perf_counter()
                    inflight.append((B.flame_dso_submit_jagged(dso, hist[i], cand[i], outs[k]), ts))
                for t, ts in inflight:
                    B.flame_dso_wait(dso, t)
                    lat.append(time.perf_counter() - ts)
                wall = time.perf_counter() - t0
                assert all(np.isfinite(o).all() for o in outs), "non-finite scores"
                lat = np.array(lat) * 1e3
                res = {"candidate_scores_per_s": float(n_scores / wall), "requests_per_s": float(len(idx) / wall),
                       "mean_latency_ms": float(lat.mean()), "p50_latency_ms": float(np.percentile(lat, 50)),
                       "p99_latency_ms": float(np.percentile(lat, 99)), "requests_in_flight": depth}
            out[f"micro_batch_{max_batch}"] = res
        finally:
            B.flame_dso_destroy(dso)
    return out


def two_stage_leg(B, wl, ws, hist, cand, one_pass_scores, steps, warmup):
    """History prefill once (per-layer K/V kept on the device), then `steps` candidate-only score calls against
    it: the two-stage paradigm of the paper's Section 5.  Reported beside the headline, never as `value`."""
    import torch
    cap = (wl.cand_offsets[1:] - wl.cand_offsets[:-1]).astype("int32")
    h = B.flame_gr_create(B.config_for(wl, kv_cache=1))
    try:
        scores = torch.zeros_like(one_pass_scores)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        B.flame_gr_prefill(h, ws, hist, wl.history_offsets, cap)       # warm-up of the prefill kernels
        torch.cuda.synchronize()
        ev[0].record()
        B.flame_gr_prefill(h, ws, hist, wl.history_offsets, cap)
        ev[1].record()
        for _ in range(warmup):
            B.flame_gr_score(h, ws, cand, wl.cand_offsets, scores)
        torch.cuda.synchronize()
        ev[2].record()
        for _ in range(steps):
            B.flame_gr_score(h, ws, cand, wl.cand_offsets, scores)
        ev[3].record()
        torch.cuda.synchronize()
        score_ms = ev[2].elapsed_time(ev[3]) / steps
        c = wl.cfg
        rows = int(wl.history_offsets[-1])
        return {"prefill_ms": ev[0].elapsed_time(ev[1]), "score_ms_per_step": score_ms,
                "scores_per_s_with_cached_history": scores.numel() / (score_ms * 1e-3),
                "bit_equal_to_one_pass": bool(torch.equal(scores, one_pass_scores)),
                "cached_kv_bytes_used": 2 * c.n_layers * rows * c.d_model * 2, "steps": steps}
    finally:
        B.flame_gr_destroy(h)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="production", help="tiny_f32 | uniform | jagged | long | production")
    ap.add_argument("--streams", type=int, default=0, help="internal stream groups of the batcher (0/1 = caller's stream)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-latency", action="store_true")
    ap.add_argument("--no-two-stage", action="store_true")
    ap.add_argument("--no-mixed-traffic", action="store_true")
    ap.add_argument("--no-climber", action="store_true")
    ap.add_argument("--no-serving", action="store_true")
    ap.add_argument("--no-small", action="store_true")
    ap.add_argument("--zero-embeddings", action="store_true",
                    help="timing probe: all embeddings zero (same kernels, same launches, operands that toggle no bits); the "
                         "chip's clock under matrix load depends on the operand data, and so does every time measured here")
    ap.add_argument("--executors", type=int, default=4, help="executors of the mixed-traffic orchestrator")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="before the timed region, run one plain device-to-device copy kernel of this many MiB "
                         "(a kernel of known HBM traffic for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (requests are independent; more GPUs would each run this same "
              "library on a share of the requests, with no collective). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2509_22681_amd import binding as B
    from paper_2509_22681_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    wl = W.make_workload(args.workload)
    cfg = wl.cfg
    dw, hist, cand = B.to_device(wl)
    if args.zero_embeddings:
        hist.zero_()
        cand.zero_()
    ws = B.pack_weights(dw)
    n_scores = int(wl.cand_offsets[-1])
    scores = torch.zeros(n_scores, device="cuda:0", dtype=torch.float32)
    h = B.flame_gr_create(B.config_for(wl, n_streams=args.streams))
    if args.calibration_copy_mib > 0:
        n = args.calibration_copy_mib * (1 << 20) // 4
        src = torch.ones(n, device="cuda:0", dtype=torch.float32)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                    # one elementwise copy kernel: reads n*4 bytes, writes n*4 bytes
        torch.cuda.synchronize()
        del src, dst
    try:
        for _ in range(args.warmup):
            B.flame_gr_forward(h, ws, hist, wl.history_offsets, cand, wl.cand_offsets, scores)
        torch.cuda.synchronize()
        # timed region: K forwards, per-kernel HIP events recorded on the launch stream
        B.flame_gr_debug_profile(h, True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            B.flame_gr_forward(h, ws, hist, wl.history_offsets, cand, wl.cand_offsets, scores)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        prof = B.flame_gr_debug_profile_read(h)
        B.flame_gr_debug_profile(h, False)
        assert torch.isfinite(scores).all().item(), "non-finite scores"
        # the same K steps without the per-kernel events, to show what the events cost
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            B.flame_gr_forward(h, ws, hist, wl.history_offsets, cand, wl.cand_offsets, scores)
        torch.cuda.synchronize()
        dt_plain = time.perf_counter() - t1
    finally:
        B.flame_gr_destroy(h)
    two_stage = None
    if cfg.dtype == "bf16" and not args.no_two_stage:
        two_stage = two_stage_leg(B, wl, ws, hist, cand, scores, args.steps, args.warmup)

    ms_per_step = dt / args.steps * 1e3
    flops_pruned = W.algorithmic_flops(cfg, wl.L, wl.M, pruned=True)
    flops_full = W.algorithmic_flops(cfg, wl.L, wl.M, pruned=False)
    full, last = attention_flops_per_layer(cfg, wl.L, wl.M)
    attn_ms, attn_launches = prof["attn"]
    attn_flops_per_step = (cfg.n_layers - 1) * full + last
    attn_avg_ms = attn_ms / max(attn_launches, 1)
    attn_flops_per_launch = attn_flops_per_step / cfg.n_layers
    achieved = attn_flops_per_launch / (attn_avg_ms * 1e-3) * 1e-12 if attn_avg_ms > 0 else 0.0
    traffic, traffic_note = stored_traffic(args.workload, attn_launches / max(args.steps, 1))
    measured_peak = measured_mfma_peak_tflops()
    out = {
        "metric": "candidate scores/sec + p50 request latency, 1 MI355X; % of bf16 MFMA peak",
        "value": n_scores / (dt / args.steps),
        "unit": "candidate scores/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        # arithmetic type of the MFMA path: fp16 operands with fp32 accumulation (embeddings and weights
        # are bf16 in HBM at the boundary); the fp32 workload computes in fp32
        "dtype": "f16" if cfg.dtype == "bf16" else "f32", "storage_dtype": cfg.dtype, "data": "synthetic" if not args.zero_embeddings else "synthetic lengths, ALL-ZERO embeddings (timing probe, not a result)",
        "config": {"workload": args.workload, "requests": wl.n_requests, "sum_L": int(wl.L.sum()), "sum_M": n_scores,
                   "d_model": cfg.d_model, "n_heads": cfg.n_heads, "n_layers": cfg.n_layers,
                   "batcher_streams": max(args.streams, 1)},
        "algorithmic_flops_per_step": flops_pruned,
        "algorithmic_flops_unpruned": flops_full,
        "pct_of_bf16_mfma_peak": 100.0 * flops_pruned / (dt / args.steps) / (PEAK_BF16_TFLOPS * 1e12),
        "ms_per_step_without_kernel_events": dt_plain / args.steps * 1e3,
        "kernel_ms_per_step": {k: v[0] / args.steps for k, v in prof.items()},
        "roofline": {"kernel": "attn_mfma_kernel" if cfg.dtype == "bf16" else "attn_f32_kernel",
                     "bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic,
                     "avg_launch_ms": attn_avg_ms, "launches": attn_launches,
                     "algorithmic_flops_per_launch": attn_flops_per_launch},
    }
    if traffic_note:
        out["roofline"]["traffic_note"] = traffic_note
    if measured_peak:
        # beside the published peak: what the matrix pipe sustains here on random operands (power-limited clock)
        out["measured_mfma_peak_tflops_random_data"] = measured_peak
        out["pct_of_measured_mfma_peak"] = 100.0 * flops_pruned / (dt / args.steps) / (measured_peak * 1e12)
        out["roofline"]["frac_of_measured_mfma_peak"] = achieved / measured_peak
    if not args.no_latency:
        # request mode: one executor (pure per-request compute latency), then eight executors in a closed loop
        # (handles created with latency_mode = 1: the attention kernel's configuration for batches that do not
        # fill the chip; the same loop on throughput-configured handles is reported beside it)
        out["request_latency"] = request_mode_latency(B, wl, dw, hist, cand, concurrency=1, latency_mode=1)
        out["p50_request_latency_ms"] = out["request_latency"]["p50_ms"]
        out["request_latency_throughput_configuration"] = request_mode_latency(B, wl, dw, hist, cand, concurrency=1)
        out["request_latency_4_executors"] = request_mode_latency(B, wl, dw, hist, cand, concurrency=4)
        out["request_latency_8_executors"] = request_mode_latency(B, wl, dw, hist, cand, concurrency=8)
    if two_stage is not None:
        out["two_stage"] = two_stage
    if not args.no_mixed_traffic:
        out["mixed_traffic"] = mixed_traffic_leg(B, wl, dw, n_executors=args.executors)
    if not args.no_serving and cfg.dtype == "bf16":
        out["host_serving"] = production_serving_leg(B, wl, dw)
    if not args.no_small:
        out["small_workloads"] = small_workloads_leg(B)
    if not args.no_climber:
        out["climber"] = climber_leg(B)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
