"""What fp16 operands alone cost: the oracle's arithmetic (fp64, the oracle's own functions) with a rounding to fp16
switched on at chosen places of the block (Section 2.1's [U V Q K], attention weights, attention output, gated rows)
and at the residual that feeds the projections.  Test infrastructure: it shows which part of a GPU-against-oracle
difference is the floor of 11-bit operands and which would be a defect.  With nothing switched on it is the oracle."""
import numpy as np

import oracle

SITES = "XUVQKPOG"      # X: the projections read the residual rounded to fp16; the rest: that tensor is rounded


def _rh(x):
    return np.asarray(x, np.float32).astype(np.float16).astype(np.float64)


def forward_request_rounded(cfg, weights, hist, cand, sites=SITES, on_layer=None):
    """Scores of one request; `cfg` as oracle.forward_request takes it (SiLU attention only)."""
    d, H = cfg["d_model"], cfg["n_heads"]
    dh = d // H
    hist = np.asarray(hist, np.float64).reshape(-1, d)
    cand = np.asarray(cand, np.float64).reshape(-1, d)
    L, M = len(hist), len(cand)
    X = np.concatenate([hist, cand])
    allow = oracle.allow_mask(L, M)
    bk = np.where(allow, oracle.bucket_matrix(L, M, cfg["n_buckets"], cfg["max_rel_dist"]), 0)
    alpha = cfg.get("attn_scale", 1.0)
    r = lambda name, x: _rh(x) if name in sites else x
    for l in range(cfg["n_layers"]):
        Xr = r("X", X)
        W1 = weights["w1"][l].astype(np.float64)
        b1 = weights["b1"][l].astype(np.float64)
        U, V, Q, K = (r(n, oracle.silu(Xr @ W1[p * d:(p + 1) * d].T + b1[p * d:(p + 1) * d])) for p, n in enumerate("UVQK"))
        O = np.zeros_like(X)
        for h in range(H):
            sl = slice(h * dh, (h + 1) * dh)
            S = alpha * (Q[:, sl] @ K[:, sl].T) + weights["rab"][l, h].astype(np.float64)[bk]
            O[:, sl] = r("P", np.where(allow, oracle.silu(S), 0.0)) @ V[:, sl]
        G = r("G", oracle.layernorm(r("O", O), weights["ln_g"][l], weights["ln_b"][l], cfg["ln_eps"]) * U)
        X = X + G @ weights["w2"][l].astype(np.float64).T + weights["b2"][l].astype(np.float64)
        if on_layer:
            on_layer(l)
    return X[L:] @ weights["w_s"].astype(np.float64) + float(weights["b_s"])
