"""CPU-only tests of the library's host logic (no GPU, no compute calls).

Checks that the C-ABI library loads and exports every declared symbol, and that its integer
planning (bucket table, mask, merged offsets, segment layout, descending-size split, stream
groups) agrees bit for bit with the oracle's independent implementation.
"""
import ctypes
import os
import re

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import oracle
from paper_2509_22681_amd import binding as B
from paper_2509_22681_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    inc = os.path.join(ROOT, "include")
    header = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    declared = set(re.findall(r"\b(flame_(?:gr|dso|climber)_[a-z_]+)\s*\(", header))
    assert {"flame_gr_create", "flame_gr_forward", "flame_gr_destroy", "flame_dso_create", "flame_dso_submit"} <= declared
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(B.EXPORTS) | set(B.DSO_EXPORTS) | set(B.CLIMBER_EXPORTS)


@pytest.mark.parametrize("nb,D", [(128, 128), (128, 1024), (128, 4096), (128, 8192), (512, 16384),
                                  (16, 512), (16, 256), (8, 32), (4, 4), (2, 2), (4, 8), (32, 128)])
def test_bucket_table_matches_oracle(nb, D):
    assert np.array_equal(B.flame_gr_host_bucket_table(nb, D), oracle.bucket_table(nb, D))


def test_bucket_table_rejects_bad_shapes():
    for nb, D in [(3, 8), (0, 8), (16, 4), (16, 100), (2, 8)]:
        with pytest.raises(B.FlameGRError) as e:
            B.flame_gr_host_bucket_table(nb, D)
        assert e.value.code == -1


@pytest.mark.parametrize("L,M,nb,D", [(3, 2, 8, 8), (64, 16, 128, 128), (0, 4, 16, 256), (5, 0, 16, 256),
                                      (300, 5, 16, 256), (0, 0, 4, 4)])
def test_host_mask_matches_oracle(L, M, nb, D):
    mask, bucket = B.flame_gr_host_mask(L, M, nb, D)
    assert np.array_equal(mask.astype(bool), oracle.allow_mask(L, M))
    assert np.array_equal(bucket, oracle.bucket_matrix(L, M, nb, D))


def _cfg(dtype="bf16", **kw):
    base = dict(n_layers=2, d_model=64, n_heads=2, n_buckets=16, max_rel_dist=1024, dtype=dtype,
                max_requests=64, max_total_tokens=1 << 20)
    base.update(kw)
    return B.make_config(**base)


def _check_layout(seg, ho, co, n_groups):
    """Segments tile the candidates of every request exactly once, rows are aligned and disjoint."""
    Bn = len(ho) - 1
    covered = [[] for _ in range(Bn)]
    end_prev = 0
    for s in seg:
        req, L, cb, M, row, grp = (int(v) for v in s)
        assert L == ho[req + 1] - ho[req]
        assert row % 64 == 0 and row >= end_prev
        end_prev = row + (L + 63) // 64 * 64 + (M + 63) // 64 * 64
        covered[req].append((cb, M))
        assert 0 <= grp < n_groups
    for i in range(Bn):
        assert covered[i], f"request {i} has no segment"
        pos = 0
        for cb, M in sorted(covered[i]):
            assert cb == pos
            pos += M
        assert pos == co[i + 1] - co[i]
    assert list(seg[:, 5]) == sorted(seg[:, 5])       # groups occupy contiguous row ranges


lens = st.lists(st.tuples(st.integers(0, 400), st.integers(0, 300)), min_size=0, max_size=12)


@settings(max_examples=60, deadline=None)
@given(lens, st.integers(1, 5))
def test_plan_offsets_and_layout(lm, n_streams):
    L = [a for a, _ in lm]
    M = [b for _, b in lm]
    ho = np.concatenate([[0], np.cumsum(L)]).astype(np.int32)
    co = np.concatenate([[0], np.cumsum(M)]).astype(np.int32)
    tok, seg = B.flame_gr_host_plan(_cfg(n_streams=n_streams), ho, co)
    assert np.array_equal(tok, oracle.merged_token_offsets(ho, co))
    assert len(seg) == len(L)
    _check_layout(seg, ho, co, n_streams)


def test_descending_split_routing():
    ho = np.array([0, 100, 130], np.int32)
    co = np.array([0, 250, 260], np.int32)
    tok, seg = B.flame_gr_host_plan(_cfg(max_seq_tokens=200), ho, co)
    _check_layout(seg, ho, co, 1)
    chunks = [(int(s[2]), int(s[3])) for s in seg if s[0] == 0]
    assert sorted(chunks) == [(0, 100), (100, 100), (200, 50)]          # largest first, remainder last
    assert [int(s[3]) for s in seg if s[0] == 1] == [10]
    with pytest.raises(B.FlameGRError) as e:                            # history alone fills the limit
        B.flame_gr_host_plan(_cfg(max_seq_tokens=100), ho, co)
    assert e.value.code == -2


def test_stream_groups_are_cost_balanced():
    wl = W.make_workload("production", lengths_only=True)
    cfg = B.make_config(16, 512, 8, 128, 8192, "bf16", max_requests=128, max_total_tokens=1 << 20, n_streams=4)
    _, seg = B.flame_gr_host_plan(cfg, wl.history_offsets, wl.cand_offsets)
    L, M = seg[:, 1].astype(np.float64), seg[:, 3].astype(np.float64)
    cost = 10 * (L + M) * 512 * 512 + 4 * (L * (L + 1) / 2 + M * (L + 1)) * 512
    per = np.array([cost[seg[:, 5] == g].sum() for g in range(4)])
    assert per.max() / per.min() < 1.05
    for g in range(4):                                                   # big requests first inside a group
        c = cost[seg[:, 5] == g]
        assert (np.diff(c) <= 0).all()


def test_offset_validation_codes():
    good_h, good_c = np.array([0, 5, 9], np.int32), np.array([0, 2, 2], np.int32)
    B.flame_gr_host_plan(_cfg(), good_h, good_c)
    for ho, co, code in [([1, 5, 9], [0, 2, 2], -1), ([0, 5, 4], [0, 2, 2], -1), ([0, 5, 9], [0, 2, 1], -1),
                         ([0, 5, 9], [3, 3, 3], -1)]:
        with pytest.raises(B.FlameGRError) as e:
            B.flame_gr_host_plan(_cfg(), np.array(ho, np.int32), np.array(co, np.int32))
        assert e.value.code == code
    with pytest.raises(B.FlameGRError) as e:
        B.flame_gr_host_plan(_cfg(max_requests=1), good_h, good_c)
    assert e.value.code == -2
    with pytest.raises(B.FlameGRError) as e:
        B.flame_gr_host_plan(_cfg(max_total_tokens=10), good_h, good_c)
    assert e.value.code == -2


def test_config_validation_codes():
    ho, co = np.array([0, 4], np.int32), np.array([0, 2], np.int32)
    for kw, code in [(dict(n_layers=0), -1), (dict(d_model=65), -1), (dict(n_buckets=12), -1),
                     (dict(max_rel_dist=1000), -1), (dict(dtype=7), -1), (dict(n_streams=99), -1),
                     (dict(d_model=96, n_heads=2), -5), (dict(d_model=64, n_heads=4), -5),
                     (dict(d_model=128, n_heads=1), -5), (dict(max_total_tokens=1 << 26), -5)]:
        with pytest.raises(B.FlameGRError) as e:
            B.flame_gr_host_plan(_cfg(**kw), ho, co)
        assert e.value.code == code, kw
    # the fp32 path has no such shape restrictions
    B.flame_gr_host_plan(_cfg(dtype="f32", d_model=96, n_heads=2), ho, co)
    B.flame_gr_host_plan(_cfg(dtype="f32", max_total_tokens=1 << 26), ho, co)
    B.flame_gr_host_plan(_cfg(max_total_tokens=(1 << 26) - (1 << 15)), ho, co)


def test_destroy_null_is_a_noop_and_bad_handle_is_reported():
    assert B._lib.flame_gr_destroy(None) == 0
    assert B._lib.flame_gr_forward(None, None, None, None, None, None, 0, None, None) == -4


# ------------------------------------------------------------------ two-stage layout (reserved candidate rows)
@settings(max_examples=60, deadline=None)
@given(st.lists(st.tuples(st.integers(0, 400), st.integers(0, 300), st.integers(0, 200)), min_size=0, max_size=12),
       st.integers(1, 5))
def test_reserved_plan_depends_on_capacity_only(lmc, n_streams):
    """The prefill (no candidates yet) and every later score call (any counts up to the capacity) must agree on
    each request's rows and stream group, or the candidate pass would not find the cached history."""
    L = [a for a, _, _ in lmc]
    M = [b for _, b, _ in lmc]
    cap = np.array([b + c for _, b, c in lmc], np.int32)
    ho = np.concatenate([[0], np.cumsum(L)]).astype(np.int32)
    co = np.concatenate([[0], np.cumsum(M)]).astype(np.int32)
    zero = np.zeros(len(L) + 1, np.int32)
    cfg = _cfg(n_streams=n_streams, kv_cache=1)
    pre = B.flame_gr_host_plan_reserved(cfg, ho, zero, cap)
    act = B.flame_gr_host_plan_reserved(cfg, ho, co, cap)
    assert len(pre) == len(act) == len(L)
    assert np.array_equal(pre[:, [0, 1, 2, 4, 5]], act[:, [0, 1, 2, 4, 5]])
    assert np.array_equal(act[:, 3], np.asarray(M, np.int32)[act[:, 0]]) and not act[:, 2].any()
    # rows: aligned, disjoint, with room for the whole capacity
    end_prev = 0
    for s in act:
        req, Lr, _, _, row, grp = (int(v) for v in s)
        assert row % 64 == 0 and row >= end_prev and 0 <= grp < n_streams
        end_prev = row + (Lr + 63) // 64 * 64 + (int(cap[req]) + 63) // 64 * 64
    assert list(act[:, 5]) == sorted(act[:, 5])


def test_reserved_plan_rejections():
    ho = np.array([0, 100, 130], np.int32)
    co = np.array([0, 20, 30], np.int32)
    with pytest.raises(B.FlameGRError) as e:                            # more candidates than reserved
        B.flame_gr_host_plan_reserved(_cfg(kv_cache=1), ho, co, [19, 10])
    assert e.value.code == -2
    with pytest.raises(B.FlameGRError) as e:
        B.flame_gr_host_plan_reserved(_cfg(kv_cache=1), ho, co, [20, -1])
    assert e.value.code == -1
    with pytest.raises(B.FlameGRError) as e:                            # reserved rows count against the capacity
        B.flame_gr_host_plan_reserved(_cfg(kv_cache=1, max_total_tokens=200), ho, co, [20, 60])
    assert e.value.code == -2
    with pytest.raises(B.FlameGRError) as e:                            # a reserved request is never split
        B.flame_gr_host_plan_reserved(_cfg(kv_cache=1, max_seq_tokens=110), ho, co, [20, 10])
    assert e.value.code == -5
    with pytest.raises(B.FlameGRError) as e:                            # the fp32 kernels have no two-stage path
        B.flame_gr_host_plan_reserved(_cfg(dtype="f32", kv_cache=1), ho, co, [20, 10])
    assert e.value.code == -5
    with pytest.raises(B.FlameGRError) as e:
        B.flame_gr_host_plan_reserved(_cfg(kv_cache=2), ho, co, [20, 10])
    assert e.value.code == -1
    seg = B.flame_gr_host_plan_reserved(_cfg(kv_cache=1), ho, co, [20, 10])
    assert len(seg) == 2


def test_block_ranges_match_the_oracle():
    for L in (0, 1, 7, 512, 1023, 1024):
        for nb in (1, 2, 3, 8):
            got = [B.flame_climber_block_range(L, nb, b) for b in range(nb)]
            assert got == [(s.start, s.stop) for s in oracle.block_slices(L, nb)]
    for args in ((10, 0, 0), (10, 2, 2), (-1, 2, 0)):
        with pytest.raises(B.FlameGRError):
            B.flame_climber_block_range(*args)


def test_split_batches_never_reach_the_spare_rows():
    """Key tiles are loaded whole (up to 128 rows), so the last 256 rows of the workspace must stay outside
    every plan.  Unsplit batches fit by construction; a split batch repeats its history per chunk and is
    rejected as soon as its padded rows would reach into the spare rows."""
    def pad(v):
        return (v + 63) // 64 * 64
    L, cap = 192, 256                      # every chunk: 192 history rows + up to 64 candidates = 256 padded rows
    for total in (1024, 1536, 4096):
        cfg = _cfg(max_requests=1, max_total_tokens=total, max_seq_tokens=cap)
        ws = B.flame_gr_host_workspace_rows(cfg)
        assert ws % 256 == 0 and ws >= total + 2 * 63 + 256
        accepted = rejected = 0
        for M in range(64, total - L + 1, 64):
            ho, co = np.array([0, L], np.int32), np.array([0, M], np.int32)
            try:
                _, seg = B.flame_gr_host_plan(cfg, ho, co)
            except B.FlameGRError as e:
                assert e.code == -2
                rejected += 1
                continue
            accepted += 1
            end = max(int(s[4]) + pad(int(s[1])) + pad(int(s[3])) for s in seg)
            assert end + 256 <= ws, (total, M, end, ws)
            assert end == 256 * len(seg)
        assert accepted > 0 and rejected > 0, (total, accepted, rejected)
    # the same bound for unsplit batches at the capacity limit
    cfg = _cfg(max_requests=4, max_total_tokens=1000)
    ws = B.flame_gr_host_workspace_rows(cfg)
    _, seg = B.flame_gr_host_plan(cfg, np.array([0, 1, 2, 3, 501], np.int32), np.array([0, 1, 2, 3, 499], np.int32))
    assert max(int(s[4]) + pad(int(s[1])) + pad(int(s[3])) for s in seg) + 256 <= ws
