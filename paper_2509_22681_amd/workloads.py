"""Seeded synthetic workloads for the GR forward (inputs only, no model arithmetic).

Every function here draws numbers and packs them into arrays; none of them evaluates any part
of the model.  Both the CPU oracle's tests and the HIP path's tests/bench take their inputs from
this module so that the two sides see bit-identical values.

The five named workloads stand in for the paper's traffic, which is private: a request is one
user history of length L_i plus M_i upstream candidates (the "single user, multiple items"
request of Section 1 / 3.2), the uniform case uses the *base* shape of Table 2 (512 history items,
128 candidates), and the jagged cases model the non-uniform upstream candidate counts that
Section 3.3 is about.  Value distributions are the ones the benchmark definition fixes:
embeddings N(0, 0.1^2), Xavier-uniform projection weights, relative-position bias N(0, 0.02^2).

numpy only; importing this module never loads the HIP library.
"""
from __future__ import annotations

from dataclasses import dataclass, field, asdict
from typing import Dict, Optional

import numpy as np

__all__ = [
    "GRConfig", "Workload", "make_workload", "make_custom", "WORKLOADS",
    "f32_to_bf16_bits", "bf16_bits_to_f32", "as_f64", "algorithmic_flops",
]


# ----------------------------------------------------------------------------------------------
# bf16 <-> fp32 bit packing (storage format conversion, round-to-nearest-even)
# ----------------------------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even) and return the 16-bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = (u + 0x7FFF + lsb) >> 16
    out = r.astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Expand 16-bit bf16 patterns to the fp32 values they denote (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


# ----------------------------------------------------------------------------------------------
# containers
# ----------------------------------------------------------------------------------------------
@dataclass
class GRConfig:
    n_layers: int
    d_model: int
    n_heads: int
    n_buckets: int
    max_rel_dist: int
    dtype: str = "bf16"          # "f32" | "bf16": storage type of embeddings and weights
    ln_eps: float = 1e-6
    attn_scale: float = 1.0
    attn_kind: str = "silu"      # "silu" | "softmax" (softmax: weights carry "temperature" [Lyr,H], fp32)

    def to_dict(self) -> dict:
        return asdict(self)


@dataclass
class Workload:
    """One batch of requests plus one set of model weights.

    Arrays hold the values *as the device receives them*: for dtype "bf16" every embedding and
    weight (except rab and b_s, which the boundary takes as fp32) is already rounded to bf16 and
    stored here as fp32 holding that rounded value; `bits(name)` gives the packed uint16 form.
    """
    name: str
    cfg: GRConfig
    history_offsets: np.ndarray      # int32 [B+1]
    cand_offsets: np.ndarray         # int32 [B+1]
    history_emb: np.ndarray          # f32 [sum L, d]
    cand_emb: np.ndarray             # f32 [sum M, d]
    weights: Dict[str, np.ndarray] = field(default_factory=dict)
    # w1 [Lyr,4d,d] (rows U|V|Q|K), b1 [Lyr,4d], rab [Lyr,H,n_buckets], ln_g/ln_b [Lyr,d],
    # w2 [Lyr,d,d], b2 [Lyr,d], w_s [d], b_s scalar (np.float32)

    @property
    def n_requests(self) -> int:
        return len(self.history_offsets) - 1

    @property
    def L(self) -> np.ndarray:
        return np.diff(self.history_offsets)

    @property
    def M(self) -> np.ndarray:
        return np.diff(self.cand_offsets)

    def bits(self, arr: np.ndarray) -> np.ndarray:
        return f32_to_bf16_bits(arr)

    def subset(self, idx) -> "Workload":
        """The workload restricted to the given requests (same weights), offsets rebuilt."""
        idx = list(idx)
        ho, co = self.history_offsets, self.cand_offsets
        h = [self.history_emb[ho[i]:ho[i + 1]] for i in idx]
        c = [self.cand_emb[co[i]:co[i + 1]] for i in idx]
        d = self.cfg.d_model
        hist = np.concatenate(h, 0) if h else np.zeros((0, d), np.float32)
        cand = np.concatenate(c, 0) if c else np.zeros((0, d), np.float32)
        nho = np.concatenate([[0], np.cumsum([len(x) for x in h])]).astype(np.int32)
        nco = np.concatenate([[0], np.cumsum([len(x) for x in c])]).astype(np.int32)
        return Workload(self.name + "[subset]", self.cfg, nho, nco, hist, cand, self.weights)


def as_f64(x: np.ndarray) -> np.ndarray:
    return np.asarray(x, dtype=np.float64)


# ----------------------------------------------------------------------------------------------
# generation
# ----------------------------------------------------------------------------------------------
def _round_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    a = np.asarray(a, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(a))
    return a


def _offsets(lengths) -> np.ndarray:
    return np.concatenate([[0], np.cumsum(np.asarray(lengths, dtype=np.int64))]).astype(np.int32)


def _pow2_above(n: int) -> int:
    p = 1
    while p <= n:
        p *= 2
    return p


def _draw(rng, cfg: GRConfig, L, M, *, emb_std=0.1, rab_std=0.02, bias_amp=0.0,
          affine_random=False, name="custom") -> Workload:
    """Draw order: history_emb, cand_emb, then per layer W1 (U,V,Q,K), W2, rab; then w_s;
    then (only when requested) biases and LayerNorm affine parameters; then (softmax attention only)
    the temperatures, Uniform[0.5, 2]."""
    d, H, Ly, nb = cfg.d_model, cfg.n_heads, cfg.n_layers, cfg.n_buckets
    sL, sM = int(np.sum(L)), int(np.sum(M))
    hist = (emb_std * rng.standard_normal((sL, d))).astype(np.float32)
    cand = (emb_std * rng.standard_normal((sM, d))).astype(np.float32)
    a_proj = np.sqrt(3.0 / d)                 # Xavier-uniform for a d -> d projection
    a_head = np.sqrt(6.0 / (d + 1))           # Xavier-uniform for d -> 1
    w1 = np.empty((Ly, 4 * d, d), np.float32)
    w2 = np.empty((Ly, d, d), np.float32)
    rab = np.empty((Ly, H, nb), np.float32)
    for l in range(Ly):
        for p in range(4):
            w1[l, p * d:(p + 1) * d] = rng.uniform(-a_proj, a_proj, (d, d))
        w2[l] = rng.uniform(-a_proj, a_proj, (d, d))
        rab[l] = rab_std * rng.standard_normal((H, nb))
    w_s = rng.uniform(-a_head, a_head, d).astype(np.float32)
    if bias_amp > 0:
        b1 = rng.uniform(-bias_amp, bias_amp, (Ly, 4 * d)).astype(np.float32)
        b2 = rng.uniform(-bias_amp, bias_amp, (Ly, d)).astype(np.float32)
        b_s = np.float32(rng.uniform(-bias_amp, bias_amp))
    else:
        b1 = np.zeros((Ly, 4 * d), np.float32)
        b2 = np.zeros((Ly, d), np.float32)
        b_s = np.float32(0.0)
    if affine_random:
        ln_g = rng.uniform(0.5, 1.5, (Ly, d)).astype(np.float32)
        ln_b = rng.uniform(-0.5, 0.5, (Ly, d)).astype(np.float32)
    else:
        ln_g = np.ones((Ly, d), np.float32)
        ln_b = np.zeros((Ly, d), np.float32)
    dt = cfg.dtype
    weights = dict(
        w1=_round_storage(w1, dt), b1=_round_storage(b1, dt), rab=rab,
        ln_g=_round_storage(ln_g, dt), ln_b=_round_storage(ln_b, dt),
        w2=_round_storage(w2, dt), b2=_round_storage(b2, dt),
        w_s=_round_storage(w_s, dt), b_s=b_s,
    )
    if cfg.attn_kind == "softmax":            # drawn last, so that the other values do not depend on the attention kind
        weights["temperature"] = rng.uniform(0.5, 2.0, (Ly, H)).astype(np.float32)
    return Workload(name, cfg, _offsets(L), _offsets(M), _round_storage(hist, dt),
                    _round_storage(cand, dt), weights)


def make_custom(L, M, *, d, H, n_layers, n_buckets, max_rel_dist=None, dtype="f32", seed=0,
                emb_std=0.1, rab_std=0.02, bias_amp=0.0, affine_random=False,
                ln_eps=1e-6, attn_scale=1.0, attn_kind="silu", name="custom") -> Workload:
    """A workload with explicit per-request lengths; used by stress and edge-case tests."""
    L = np.asarray(L, dtype=np.int64)
    M = np.asarray(M, dtype=np.int64)
    if max_rel_dist is None:
        max_rel_dist = _pow2_above(int(L.max()) if len(L) else 0)
    cfg = GRConfig(n_layers, d, H, n_buckets, max_rel_dist, dtype, ln_eps, attn_scale, attn_kind)
    rng = np.random.default_rng(seed)
    return _draw(rng, cfg, L, M, emb_std=emb_std, rab_std=rab_std, bias_amp=bias_amp,
                 affine_random=affine_random, name=name)


# name -> (B, L spec, M spec, d, H, layers, n_buckets, dtype)
#   L spec: int (constant) or ("uniform", lo, hi);  M spec: int or ("zipf", s, lo, hi)
WORKLOADS = {
    "tiny_f32":   dict(B=1,   L=64,                     M=16,                       d=64,  H=2, layers=2,  n_buckets=128, dtype="f32"),
    "uniform":    dict(B=32,  L=512,                    M=128,                      d=256, H=4, layers=4,  n_buckets=128, dtype="bf16"),
    "jagged":     dict(B=64,  L=("uniform", 256, 2048), M=("zipf", 1.2, 16, 1024),  d=512, H=8, layers=8,  n_buckets=128, dtype="bf16"),
    "long":       dict(B=16,  L=8192,                   M=512,                      d=512, H=8, layers=8,  n_buckets=512, dtype="bf16"),
    "production": dict(B=128, L=("uniform", 1024, 4096), M=("zipf", 1.1, 32, 2000), d=512, H=8, layers=16, n_buckets=128, dtype="bf16"),
    # the production shape with the softmax-with-temperature attention of the paper's own model (same lengths and
    # values: the temperatures are drawn last)
    "production_softmax": dict(B=128, L=("uniform", 1024, 4096), M=("zipf", 1.1, 32, 2000), d=512, H=8, layers=16, n_buckets=128,
                               dtype="bf16", attn_kind="softmax"),
}


def make_workload(name: str, seed: int = 0, lengths_only: bool = False) -> Optional[Workload]:
    """One of the named benchmark workloads (the five of the benchmark definition and the softmax variant of the last).

    Lengths: L_i constant or Uniform[lo, hi] (inclusive); M_i constant or an unbounded Zipf(s)
    draw clipped to [lo, hi].  Lengths are drawn first (L then M) from default_rng(seed), then the
    values in the order `_draw` documents.  max_rel_dist is the smallest power of two above the
    longest history the workload's length range allows, so the bias table never clamps.
    """
    s = WORKLOADS[name]
    rng = np.random.default_rng(seed)
    B = s["B"]
    Ls, Ms = s["L"], s["M"]
    L = np.full(B, Ls, np.int64) if isinstance(Ls, int) else rng.integers(Ls[1], Ls[2] + 1, B)
    M = np.full(B, Ms, np.int64) if isinstance(Ms, int) else np.clip(rng.zipf(Ms[1], B), Ms[2], Ms[3])
    L_hi = Ls if isinstance(Ls, int) else Ls[2]
    cfg = GRConfig(s["layers"], s["d"], s["H"], s["n_buckets"], _pow2_above(L_hi), s["dtype"],
                   attn_kind=s.get("attn_kind", "silu"))
    if lengths_only:
        return Workload(name, cfg, _offsets(L), _offsets(M), np.zeros((0, s["d"]), np.float32),
                        np.zeros((0, s["d"]), np.float32), {})
    return _draw(rng, cfg, L, M, name=name)


# ----------------------------------------------------------------------------------------------
# work accounting (counts only; used for the roofline denominator)
# ----------------------------------------------------------------------------------------------
def algorithmic_flops(cfg: GRConfig, L, M, pruned: bool = True) -> float:
    """Multiply-add work (2 flop per MAC) the forward must do for these request lengths.

    Per request and layer: 10*N*d^2 for the two projections (UVQK 8, output 2) and 4*P*d for the
    two attention products over the P allowed (query, key) pairs.  With `pruned`, the last layer
    counts only what the scores depend on: K,V for history rows, U,V,Q,K for candidate rows,
    candidate query rows only, output projection of candidate rows only.
    """
    L = np.asarray(L, dtype=np.float64)
    M = np.asarray(M, dtype=np.float64)
    d, Ly = float(cfg.d_model), cfg.n_layers
    N = L + M
    P = L * (L + 1) / 2 + M * (L + 1)
    full = 10 * N * d * d + 4 * P * d
    head = 2 * M.sum() * d
    if not pruned:
        return float(Ly * full.sum() + head)
    last = 4 * L * d * d + 8 * M * d * d + 4 * M * (L + 1) * d + 2 * M * d * d
    return float((Ly - 1) * full.sum() + last.sum() + head)
