"""CPU oracle for the generative-recommendation (GR) forward.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain definition that the HIP library is checked against.  Only tests, the
smoke check and the benchmark's CPU-baseline leg may import it; the product path never does, and it
imports nothing from the product package.  All arithmetic is float64 numpy; inputs are whatever
values the device receives, up-cast exactly.

What is computed (one request = a user history of L items followed by M candidate items):

* Problem statement - Section 1 ("single user, multiple items" per request), Section 2.1
  (candidates are appended after the user's behaviour sequence), Section 3.2 (a customised
  attention mask lets all candidates be scored in one pass, independently of each other) and
  Section 3.3 (the number of candidates per request varies).
* Block arithmetic - the paper gives no equations.  The block is the pointwise-SiLU sequence
  transducer the paper cites for its mask design (Section 3.2), as fixed by the benchmark
  definition:  [U V Q K] = silu(X W1^T + b1);  per head  O_r = sum_c silu(alpha <Q_r,K_c> +
  rab[bucket(pos_r - pos_c)]) V_c  over the allowed keys c;  X <- X + (LayerNorm(O) * U) W2^T + b2;
  score = <w_s, X_cand> + b_s.

Readings taken where the sources are silent (each is also listed in the design document):
  - history rows attend causally, own position included; candidate rows attend to the whole
    history and to themselves only;
  - every candidate sits at position L (the next slot), which is what makes the scores invariant
    under a permutation of the candidates;
  - no attention normaliser (no 1/n, no 1/sqrt(d_h)); alpha is a configuration scalar;
  - LayerNorm over the full model width with biased variance;
  - the relative-position bucket function below (integer only).

Softmax variant (the paper's own model, Section 2.1: Transformer blocks with "an adaptive temperature
coefficient ... before softmax", the user sequence cut into N_b sub-sequences that independent blocks
process, every candidate appended to each sub-sequence, block outputs joined by a "bit-wise gating
fusion module", task probabilities from the "expert module of the top-level multi-layer
perceptron").  The paper gives prose only; the readings taken here:
  - cfg["attn_kind"] == "softmax": the attention weights of a row are softmax over its allowed keys of
    (alpha <Q_r,K_c> + rab[bucket]) / tau[l,h], tau a positive learned scalar per layer and head
    (w["temperature"]); everything else in the block is unchanged;
  - sub-sequence b of N_b is the contiguous slice [floor(b L / N_b), floor((b+1) L / N_b)) of the history,
    positions restart at 0 inside a slice; block b has its own weights and sees all candidates;
  - fusion: with H_b [M,d] the candidates' final residual rows of block b and C = [H_0 | ... | H_{N_b-1}],
    g_b = sigmoid(C Wg_b^T + cg_b) elementwise over the d features ("bit-wise" = per feature), F = sum_b g_b * H_b;
  - head: T tasks, p_t = sigmoid(<v_t, relu(F A_t^T + a_t)> + c_t) with expert width E.

Parity status: the paper prints no model output, so against the paper itself this oracle is
"parity unpinned".  It is pinned instead (tests/test_oracle_*.py) by a hand-worked case, by the
scalar-loop transcription `forward_request_loops` on tiny inputs, by closed forms that reduce to a
GEMV / prefix sum / plain LayerNorm, and by the independence, causality and masking invariants.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional

import numpy as np

F64 = np.float64


# ----------------------------------------------------------------------------------------------
# elementary pieces
# ----------------------------------------------------------------------------------------------
def silu(x):
    """silu(x) = x / (1 + exp(-x)), evaluated without overflow for large |x|."""
    x = np.asarray(x, dtype=F64)
    e = np.exp(-np.abs(x))                       # in (0, 1]
    sig = np.where(x >= 0, 1.0 / (1.0 + e), e / (1.0 + e))
    return x * sig


def layernorm(o, gamma, beta, eps):
    """Row-wise LayerNorm over the last axis, biased variance."""
    o = np.asarray(o, dtype=F64)
    mu = o.mean(axis=-1, keepdims=True)
    var = ((o - mu) ** 2).mean(axis=-1, keepdims=True)
    return (o - mu) / np.sqrt(var + eps) * gamma + beta


def _ilog2(n: int) -> int:
    assert n > 0 and (n & (n - 1)) == 0, "power of two expected"
    return n.bit_length() - 1


def bucket_scalar(delta: int, n_buckets: int, max_rel_dist: int) -> int:
    """Relative-position bucket of a distance delta >= 0 (integers only).

    The near half of the table is exact: delta < E = n_buckets/2 maps to itself.  The far half is
    log-spaced: each octave [2^e, 2^(e+1)) between E and max_rel_dist is cut into 2^m equal
    sub-buckets, with m the largest value for which all octaves fit into the far half.  Distances
    at or beyond max_rel_dist share the last used bucket.
    """
    E = n_buckets // 2
    e0, e1 = _ilog2(E), _ilog2(max_rel_dist)
    delta = min(int(delta), max_rel_dist - 1)
    if delta < E:
        return delta
    n_oct = max(e1 - e0, 0)
    m = e0
    while n_oct * (1 << m) > E:
        m -= 1
    e = delta.bit_length() - 1
    return E + (e - e0) * (1 << m) + ((delta - (1 << e)) >> (e - m))


def bucket_table(n_buckets: int, max_rel_dist: int) -> np.ndarray:
    """bucket_scalar for every delta in [0, max_rel_dist)."""
    return np.array([bucket_scalar(t, n_buckets, max_rel_dist) for t in range(max_rel_dist)],
                    dtype=np.int32)


def positions(L: int, M: int) -> np.ndarray:
    """Position index of each token: history token t sits at t, every candidate at L."""
    return np.concatenate([np.arange(L, dtype=np.int64), np.full(M, L, dtype=np.int64)])


def allow_mask(L: int, M: int) -> np.ndarray:
    """Boolean [N, N]: may query row r look at key column c?"""
    N = L + M
    r = np.arange(N)[:, None]
    c = np.arange(N)[None, :]
    hist_row = r < L
    return np.where(hist_row, c <= r, (c < L) | (c == r))


def bucket_matrix(L: int, M: int, n_buckets: int, max_rel_dist: int) -> np.ndarray:
    """int32 [N, N] bucket of pos[r]-pos[c]; entries of disallowed pairs are set to -1."""
    pos = positions(L, M)
    delta = pos[:, None] - pos[None, :]
    tab = bucket_table(n_buckets, max_rel_dist)
    out = np.full(delta.shape, -1, dtype=np.int32)
    ok = allow_mask(L, M)
    dd = np.minimum(delta[ok], max_rel_dist - 1)
    out[ok] = tab[dd]
    return out


def merged_token_offsets(history_offsets, cand_offsets) -> np.ndarray:
    """Start of each request in the merged token order (history then candidates, per request)."""
    return (np.asarray(history_offsets, np.int64) + np.asarray(cand_offsets, np.int64)).astype(np.int32)


# ----------------------------------------------------------------------------------------------
# the forward, vectorised per request
# ----------------------------------------------------------------------------------------------
def masked_softmax(z, allow):
    """Row-wise softmax of z over the entries where allow is True (0 elsewhere); every row of `allow`
    has at least one True."""
    z = np.where(allow, np.asarray(z, F64), -np.inf)
    z = z - z.max(axis=-1, keepdims=True)
    e = np.where(allow, np.exp(z), 0.0)
    return e / e.sum(axis=-1, keepdims=True)


def forward_request(cfg: dict, w: Dict[str, np.ndarray], hist: np.ndarray, cand: np.ndarray,
                    stages: Optional[List[dict]] = None, hidden: bool = False) -> np.ndarray:
    """Scores of one request.  hist [L,d], cand [M,d]; returns [M] (or, with hidden=True, the
    candidates' final residual rows [M,d] instead of their scores).

    If `stages` is a list, one dict per layer with the tensors U,V,Q,K,O,X (X after the residual)
    is appended to it.  cfg["attn_kind"] ("silu", the default, or "softmax") selects the attention
    weights (see the file header).
    """
    d, H, Ly = cfg["d_model"], cfg["n_heads"], cfg["n_layers"]
    nb, D = cfg["n_buckets"], cfg["max_rel_dist"]
    eps, alpha = cfg["ln_eps"], cfg["attn_scale"]
    softmax = cfg.get("attn_kind", "silu") == "softmax"
    dh = d // H
    L, M = hist.shape[0], cand.shape[0]
    X = np.concatenate([np.asarray(hist, F64).reshape(L, d), np.asarray(cand, F64).reshape(M, d)], 0)
    N = L + M
    allow = allow_mask(L, M)
    bkt = bucket_matrix(L, M, nb, D)
    bkt_safe = np.where(allow, bkt, 0)
    for l in range(Ly):
        Z = X @ np.asarray(w["w1"][l], F64).T + np.asarray(w["b1"][l], F64)
        A = silu(Z)
        U, V, Q, K = A[:, 0:d], A[:, d:2 * d], A[:, 2 * d:3 * d], A[:, 3 * d:4 * d]
        O = np.zeros((N, d), F64)
        for h in range(H):
            sl = slice(h * dh, (h + 1) * dh)
            S = alpha * (Q[:, sl] @ K[:, sl].T) + np.asarray(w["rab"][l, h], F64)[bkt_safe]
            if softmax:
                Wgt = masked_softmax(S / float(w["temperature"][l, h]), allow)
            else:
                Wgt = np.where(allow, silu(S), 0.0)
            O[:, sl] = Wgt @ V[:, sl]
        Y = layernorm(O, np.asarray(w["ln_g"][l], F64), np.asarray(w["ln_b"][l], F64), eps) * U
        X = X + Y @ np.asarray(w["w2"][l], F64).T + np.asarray(w["b2"][l], F64)
        if stages is not None:
            stages.append(dict(U=U, V=V, Q=Q, K=K, O=O, X=X.copy()))
    if hidden:
        return X[L:].copy()
    return X[L:] @ np.asarray(w["w_s"], F64) + float(w["b_s"])


def forward(cfg: dict, w: Dict[str, np.ndarray], history_emb, history_offsets, cand_emb,
            cand_offsets, stages: Optional[List[List[dict]]] = None, hidden: bool = False) -> np.ndarray:
    """Scores of a jagged batch, in cand_offsets order (hidden=True: the candidates' final residual
    rows [sum M, d]).  Requests are independent."""
    ho = np.asarray(history_offsets, np.int64)
    co = np.asarray(cand_offsets, np.int64)
    B = len(ho) - 1
    assert len(co) - 1 == B
    n_out = int(co[-1]) if B >= 0 and len(co) else 0
    scores = np.zeros((n_out, cfg["d_model"]) if hidden else n_out, F64)
    for i in range(B):
        st = [] if stages is not None else None
        scores[co[i]:co[i + 1]] = forward_request(
            cfg, w, history_emb[ho[i]:ho[i + 1]], cand_emb[co[i]:co[i + 1]], st, hidden)
        if stages is not None:
            stages.append(st)
    return scores


# ----------------------------------------------------------------------------------------------
# sub-sequence blocks, gating fusion and the task head (Section 2.1; readings in the file header)
# ----------------------------------------------------------------------------------------------
def sigmoid(x):
    x = np.asarray(x, dtype=F64)
    e = np.exp(-np.abs(x))
    return np.where(x >= 0, 1.0 / (1.0 + e), e / (1.0 + e))


def block_slices(L: int, n_blocks: int) -> List[slice]:
    """Contiguous sub-sequences of a history of L items: block b takes [floor(b L / N_b), floor((b+1) L / N_b))."""
    return [slice(b * L // n_blocks, (b + 1) * L // n_blocks) for b in range(n_blocks)]


def fuse_and_score(head: Dict[str, np.ndarray], hidden_blocks: List[np.ndarray]) -> np.ndarray:
    """hidden_blocks: N_b arrays [M,d].  Returns task probabilities [M,T].
    head: wg [N_b][d][N_b*d], cg [N_b][d], a_w [T][E][d], a_b [T][E], v [T][E], c [T]."""
    Hs = [np.asarray(h, F64) for h in hidden_blocks]
    C = np.concatenate(Hs, axis=1)
    F = np.zeros_like(Hs[0])
    for b, Hb in enumerate(Hs):
        F += sigmoid(C @ np.asarray(head["wg"][b], F64).T + np.asarray(head["cg"][b], F64)) * Hb
    T = len(head["c"])
    out = np.zeros((F.shape[0], T), F64)
    for t in range(T):
        E = np.maximum(F @ np.asarray(head["a_w"][t], F64).T + np.asarray(head["a_b"][t], F64), 0.0)
        out[:, t] = sigmoid(E @ np.asarray(head["v"][t], F64) + float(head["c"][t]))
    return out


def climber_request(cfg: dict, block_weights: List[Dict[str, np.ndarray]], head: Dict[str, np.ndarray],
                    hist: np.ndarray, cand: np.ndarray) -> np.ndarray:
    """Task probabilities [M,T] of one request through N_b = len(block_weights) independent blocks."""
    hist = np.asarray(hist)
    hs = [forward_request(cfg, wb, hist[sl], cand, hidden=True)
          for wb, sl in zip(block_weights, block_slices(hist.shape[0], len(block_weights)))]
    return fuse_and_score(head, hs)


# ----------------------------------------------------------------------------------------------
# the same definition as scalar loops (tiny inputs only).  Of the code above it calls only `bucket_scalar`
# (pinned on its own by hand-computed values); mask, positions, SiLU, softmax and LayerNorm are written out again
# ----------------------------------------------------------------------------------------------
def forward_request_loops(cfg: dict, w, hist, cand) -> List[float]:
    d, H, Ly = cfg["d_model"], cfg["n_heads"], cfg["n_layers"]
    nb, D = cfg["n_buckets"], cfg["max_rel_dist"]
    eps, alpha = cfg["ln_eps"], cfg["attn_scale"]
    softmax = cfg.get("attn_kind", "silu") == "softmax"
    dh = d // H
    L, M = len(hist), len(cand)
    N = L + M
    X = [[float(v) for v in row] for row in list(hist) + list(cand)]

    def s(x):
        return x / (1.0 + math.exp(-x)) if x > -700 else 0.0

    for l in range(Ly):
        W1, b1 = w["w1"][l], w["b1"][l]
        A = [[s(sum(X[t][k] * float(W1[j][k]) for k in range(d)) + float(b1[j]))
              for j in range(4 * d)] for t in range(N)]
        O = [[0.0] * d for _ in range(N)]
        for r in range(N):
            pr = r if r < L else L
            keys = [c for c in range(N) if (c <= r if r < L else (c < L or c == r))]
            for h in range(H):
                logit = []
                for c in keys:
                    pc = c if c < L else L
                    bk = bucket_scalar(pr - pc, nb, D)
                    dot = 0.0
                    for k in range(dh):
                        dot += A[r][2 * d + h * dh + k] * A[c][3 * d + h * dh + k]
                    logit.append(alpha * dot + float(w["rab"][l][h][bk]))
                if softmax:
                    tau = float(w["temperature"][l][h])
                    top = max(v / tau for v in logit)
                    ex = [math.exp(v / tau - top) for v in logit]
                    tot = sum(ex)
                    wgts = [e / tot for e in ex]
                else:
                    wgts = [s(v) for v in logit]
                for c, wgt in zip(keys, wgts):
                    for k in range(dh):
                        O[r][h * dh + k] += wgt * A[c][d + h * dh + k]
        for r in range(N):
            mu = sum(O[r]) / d
            var = sum((v - mu) ** 2 for v in O[r]) / d
            inv = 1.0 / math.sqrt(var + eps)
            Y = [((O[r][k] - mu) * inv * float(w["ln_g"][l][k]) + float(w["ln_b"][l][k])) * A[r][k]
                 for k in range(d)]
            for j in range(d):
                X[r][j] += sum(Y[k] * float(w["w2"][l][j][k]) for k in range(d)) + float(w["b2"][l][j])
    return [sum(float(w["w_s"][k]) * X[L + j][k] for k in range(d)) + float(w["b_s"])
            for j in range(M)]
