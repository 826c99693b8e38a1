"""The rounding emulator of tests/fp16_floor.py against the oracle: with no rounding switched on it is the oracle; with
roundings on, every site moves the scores, by about what an 11-bit operand should."""
import numpy as np

import oracle
from paper_2509_22681_amd import workloads as W
from tests.fp16_floor import SITES, forward_request_rounded


def small():
    return W.make_custom([150, 0, 37], [40, 9, 0], d=64, H=2, n_layers=3, n_buckets=32, dtype="bf16", seed=5,
                         emb_std=1.0, rab_std=1.0, bias_amp=0.5, affine_random=True, attn_scale=0.7, name="floor")


def request(wl, i):
    ho, co = wl.history_offsets, wl.cand_offsets
    return wl.history_emb[ho[i]:ho[i + 1]], wl.cand_emb[co[i]:co[i + 1]]


def test_without_roundings_it_is_the_oracle():
    wl = small()
    cfg = wl.cfg.to_dict()
    for i in range(wl.n_requests):
        hist, cand = request(wl, i)
        want = oracle.forward_request(cfg, wl.weights, hist, cand)
        got = forward_request_rounded(cfg, wl.weights, hist, cand, sites="")
        assert got.shape == want.shape
        if len(want):
            assert np.max(np.abs(got - want)) <= 1e-12 * max(1.0, np.max(np.abs(want)))


def test_every_site_moves_the_scores_by_a_few_ulp_of_fp16():
    wl = small()
    cfg = wl.cfg.to_dict()
    hist, cand = request(wl, 0)
    want = oracle.forward_request(cfg, wl.weights, hist, cand)
    rms = np.sqrt(np.mean(want * want))
    each = {}
    for s in SITES:
        e = forward_request_rounded(cfg, wl.weights, hist, cand, sites=s) - want
        each[s] = np.sqrt(np.mean(e * e)) / rms
        assert 2e-5 < each[s] < 5e-3, (s, each[s])          # 2^-12 is 2.4e-4
    e = forward_request_rounded(cfg, wl.weights, hist, cand) - want
    both = np.sqrt(np.mean(e * e)) / rms
    quad = np.sqrt(sum(v * v for v in each.values()))
    assert 0.5 * quad < both < 2.0 * quad, (both, quad, each)   # the sites add roughly in quadrature
