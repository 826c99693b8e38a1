"""Host logic of the request orchestrator: the descending-size split routing (Section 3.3 of the paper), checked
without a GPU against its stated properties, an independent brute force over the rule's choices, and worked cases."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from paper_2509_22681_amd import binding as B

PAPER_PROFILES = [128, 256, 512, 1024]


def cost(L, p, d):
    N = L + p
    P = L * (L + 1) // 2 + p * (L + 1)
    return 10 * N * d * d + 4 * P * d


def brute_force_remainder(prof, L, d, r):
    """Cheapest way to serve r < max(prof) candidates with a descending run of full profiles closed by at most one
    padded chunk: enumerate every non-increasing sequence of profiles whose full chunks stay below r."""
    best = None
    def rec(rem, seq, ceiling):
        nonlocal best
        if rem == 0:
            c = sum(cost(L, p, d) for p in seq)
            if best is None or c < best:
                best = c
            return
        ups = [p for p in prof if p >= rem]
        if ups:
            c = sum(cost(L, p, d) for p in seq) + cost(L, ups[0], d)
            if best is None or c < best:
                best = c
        for p in prof:
            if p < rem and p <= ceiling:
                rec(rem - p, seq + [p], p)
    rec(r, [], max(prof))
    return best


@settings(max_examples=300, deadline=None)
@given(st.lists(st.integers(1, 300), min_size=1, max_size=5, unique=True), st.integers(0, 2000), st.integers(1, 1500),
       st.sampled_from([8, 64, 512]))
def test_route_properties(prof, L, M, d):
    prof = sorted(prof)
    chunks = B.flame_dso_route(prof, L, d, M)
    sizes = [prof[p] for p, _ in chunks]
    counts = [c for _, c in chunks]
    assert sum(counts) == M                                   # every candidate exactly once
    assert all(1 <= c <= s for c, s in zip(counts, sizes))    # a chunk fits its profile
    assert sizes == sorted(sizes, reverse=True)               # descending order
    assert all(c == s for c, s in zip(counts[:-1], sizes[:-1]))   # only the last chunk may be padded
    top = prof[-1]
    assert sizes[:M // top] == [top] * (M // top)             # the largest profile while it fits
    # the remainder is served at the least cost the rule allows
    rest = sizes[M // top:]
    r = M % top
    if r:
        greedy_family = []
        rem = r
        # the rule only ever takes the LARGEST profile below the remainder when it splits
        def walk(rem, acc):
            ups = [p for p in prof if p >= rem]
            if ups:
                greedy_family.append(acc + [ups[0]])
            downs = [p for p in prof if p < rem]
            if downs:
                walk(rem - downs[-1], acc + [downs[-1]])
        walk(rem, [])
        want = min(sum(cost(L, p, d) for p in seq) for seq in greedy_family)
        assert sum(cost(L, p, d) for p in rest) == want
        assert want >= brute_force_remainder(prof, L, d, r)   # (the full search may only be cheaper or equal)
    else:
        assert rest == []


def test_route_worked_cases():
    P = PAPER_PROFILES
    for M in P:                                               # the paper's mixed traffic: exact hits
        assert B.flame_dso_route(P, 1024, 512, M) == [(P.index(M), M)]
    # a long history makes one padded chunk cheaper than re-running the history for a second chunk
    assert B.flame_dso_route(P, 1024, 512, 700) == [(3, 700)]
    assert B.flame_dso_route(P, 1024, 512, 130) == [(1, 130)]
    assert B.flame_dso_route(P, 1024, 512, 2500) == [(3, 1024), (3, 1024), (2, 452)]
    assert B.flame_dso_route(P, 1024, 512, 1) == [(0, 1)]
    # with no history the rows of the padding dominate: split into full chunks as far as it pays
    assert B.flame_dso_route(P, 0, 512, 640) == [(2, 512), (0, 128)]
    assert B.flame_dso_route(P, 0, 512, 130) == [(1, 130)]     # equal cost: the fewer chunks win
    # implicit shapes: any count up to the largest profile in one piece
    assert B.flame_dso_route(P, 1024, 512, 700, explicit_shapes=False) == [(-1, 700)]
    assert B.flame_dso_route(P, 1024, 512, 2500, explicit_shapes=False) == [(-1, 1024), (-1, 1024), (-1, 452)]
    assert B.flame_dso_route(P, 1024, 512, 0) == []


def test_route_rejects_bad_profiles():
    for prof in ([], [0, 4], [4, 4], [8, 4], list(range(1, 18))):
        with pytest.raises(B.FlameGRError) as e:
            B.flame_dso_route(prof, 10, 64, 5)
        assert e.value.code == -1
    with pytest.raises(B.FlameGRError) as e:
        B.flame_dso_route([4, 8], 10, 64, -1)
    assert e.value.code == -1
