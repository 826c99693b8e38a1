"""Oracle scores for the named benchmark workloads, stored as text fixtures.

The expected values are produced by `oracle.forward_request` and by nothing else.  Because the big
workloads take minutes of fp64 numpy per request (five minutes for one 8192-token history), the
results are kept as text files under tests/golden/oracle_scores/, one per request, keyed by a hash
of the exact inputs (configuration, the request's embeddings, all weights).  This script is the only
writer of those files:

    python tests/oracle_cache.py [--jobs J] [workload ...]

(`--jobs J` spreads the requests of a workload over J single-threaded worker processes, most expensive
request first; the arithmetic is `oracle.forward_request` either way.)

A file whose key does not match the regenerated inputs is simply not found, and the tests then
compute the values in place.
"""
from __future__ import annotations

import hashlib
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2509_22681_amd import workloads as W  # noqa: E402

CACHE_DIR = os.path.join(ROOT, "tests", "golden", "oracle_scores")

# requests whose oracle scores are compared at the full benchmark sizes (all requests where None)
SAMPLED = {
    "tiny_f32": None,
    "uniform": None,
    "jagged": None,
    "long": None,
    "production": None,
    "production_softmax": "spread",
}


def sample_requests(wl: W.Workload, name: str):
    spec = SAMPLED[name]
    if spec is None:
        return list(range(wl.n_requests))
    if spec == "spread":
        L, M = wl.L.astype(np.int64), wl.M.astype(np.int64)
        cost = 10 * (L + M) * wl.cfg.d_model + 4 * (L * (L + 1) // 2 + M * (L + 1))
        order = np.argsort(cost, kind="stable")
        picks = [int(order[0]), int(order[len(order) // 2]), int(order[-1])]
        rng = np.random.default_rng(12345)
        for r in rng.permutation(wl.n_requests):
            if int(r) not in picks:
                picks.append(int(r))
            if len(picks) == 5:
                break
        return picks
    return list(spec)


_weights_digest = {}        # id(weights dict) -> (the dict itself, digest): the reference keeps the id from being reused


def _key(wl: W.Workload, i: int) -> str:
    memo = _weights_digest.get(id(wl.weights))
    if memo is None or memo[0] is not wl.weights:
        hw = hashlib.sha1()
        for k in sorted(wl.weights):
            hw.update(np.ascontiguousarray(wl.weights[k]).tobytes())
        if len(_weights_digest) >= 8:       # bounded: the oldest entry goes
            _weights_digest.pop(next(iter(_weights_digest)))
        memo = _weights_digest[id(wl.weights)] = (wl.weights, hw.digest())
    wd = memo[1]
    h = hashlib.sha1(wd)
    ho, co = wl.history_offsets, wl.cand_offsets
    cfg = wl.cfg.to_dict()
    if cfg.get("attn_kind") == "silu":      # the default kind is not part of the key (fixtures older than the field stay valid)
        del cfg["attn_kind"]
    h.update(repr(sorted(cfg.items())).encode())
    h.update(np.ascontiguousarray(wl.history_emb[ho[i]:ho[i + 1]]).tobytes())
    h.update(np.ascontiguousarray(wl.cand_emb[co[i]:co[i + 1]]).tobytes())
    return h.hexdigest()[:20]


def request_scores(wl: W.Workload, i: int, verbose: bool = False) -> np.ndarray:
    """Oracle scores of request i of a workload (cached)."""
    path = os.path.join(CACHE_DIR, f"{wl.name}_req{i}_{_key(wl, i)}.txt")
    if os.path.exists(path):
        return np.loadtxt(path, dtype=np.float64, ndmin=1)
    t = time.time()
    ho, co = wl.history_offsets, wl.cand_offsets
    if (ho[i + 1] - ho[i]) + (co[i + 1] - co[i]) > 2048:      # minutes of CPU work: never silent
        print(f"  no stored oracle scores for {wl.name} request {i} ({os.path.basename(path)}): computing", flush=True)
    s = oracle.forward_request(wl.cfg.to_dict(), wl.weights, wl.history_emb[ho[i]:ho[i + 1]],
                               wl.cand_emb[co[i]:co[i + 1]])
    if verbose:
        print(f"  oracle {wl.name} request {i}: L={ho[i + 1] - ho[i]} M={co[i + 1] - co[i]} "
              f"{time.time() - t:.1f}s", flush=True)
    try:
        os.makedirs(CACHE_DIR, exist_ok=True)
        tmp = path + f".tmp{os.getpid()}"
        np.savetxt(tmp, s, fmt="%.17g")
        os.replace(tmp, path)
    except OSError:
        pass
    return s


_worker_wl = {}


def _worker(task):
    name, i = task
    wl = _worker_wl.get(name)
    if wl is None:
        _worker_wl.clear()
        wl = _worker_wl[name] = W.make_workload(name)
    request_scores(wl, i, verbose=True)
    return i


def main(names, jobs=1):
    for name in names:
        if jobs <= 1:
            wl = W.make_workload(name)
            for i in sample_requests(wl, name):
                request_scores(wl, i, verbose=True)
            continue
        import multiprocessing as mp
        lens = W.make_workload(name, lengths_only=True)
        L, M = lens.L.astype(np.int64), lens.M.astype(np.int64)
        todo = sorted(sample_requests(lens, name), key=lambda i: -int((L[i] + M[i]) ** 2))
        for v in ("OMP_NUM_THREADS", "OPENBLAS_NUM_THREADS", "MKL_NUM_THREADS"):
            os.environ[v] = "1"                    # inherited by the spawned workers
        with mp.get_context("spawn").Pool(jobs) as pool:
            for _ in pool.imap_unordered(_worker, [(name, i) for i in todo], chunksize=1):
                pass


if __name__ == "__main__":
    args = sys.argv[1:]
    jobs = 1
    if args and args[0] == "--jobs":
        jobs = int(args[1])
        args = args[2:]
    main(args or list(SAMPLED), jobs)
