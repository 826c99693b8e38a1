"""ctypes binding of libflame_gr.so: argument marshalling only.

Function names mirror the C ABI (include/flame_gr.h).  PyTorch tensors are accepted wherever the
ABI takes a device pointer; numpy arrays wherever it takes a host pointer.  Nothing here computes
any part of the forward, and nothing falls back to another implementation: if the library has not
been built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import numpy as np
# PyTorch provides device memory and streams.  It must be imported before the library is loaded so
# that both resolve libamdhip64.so.7 to the one HIP runtime PyTorch bundles: two HIP runtimes in one
# process do not both see the device.
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflame_gr.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
        "or python paper_2509_22681_amd/build.py)")

_lib = C.CDLL(LIB_PATH)

FLAME_GR_F32, FLAME_GR_BF16 = 0, 1
FLAME_GR_ATTN_SILU, FLAME_GR_ATTN_SOFTMAX = 0, 1
STATUS = {0: "OK", -1: "INVALID_ARGUMENT", -2: "CAPACITY_EXCEEDED", -3: "HIP_ERROR", -4: "BAD_HANDLE",
          -5: "UNSUPPORTED"}
KERNEL_KINDS = ("assemble", "bias", "uvqk", "attn", "ln_gate", "outproj", "score")


class flame_gr_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("n_buckets", C.c_int32), ("max_rel_dist", C.c_int32), ("dtype", C.c_int32),
                ("ln_eps", C.c_float), ("attn_scale", C.c_float),
                ("max_requests", C.c_int32), ("max_total_tokens", C.c_int32),
                ("max_seq_tokens", C.c_int32), ("n_streams", C.c_int32), ("attn_kind", C.c_int32),
                ("kv_cache", C.c_int32), ("latency_mode", C.c_int32), ("weights_static", C.c_int32)]


class flame_gr_weights(C.Structure):
    _fields_ = [("w1", C.c_void_p), ("b1", C.c_void_p), ("rab", C.c_void_p), ("ln_g", C.c_void_p),
                ("ln_b", C.c_void_p), ("w2", C.c_void_p), ("b2", C.c_void_p), ("w_s", C.c_void_p),
                ("b_s", C.c_float), ("temperature", C.c_void_p)]


_i32p = C.POINTER(C.c_int32)
_lib.flame_gr_create.argtypes = [C.POINTER(flame_gr_config), C.POINTER(C.c_void_p)]
_lib.flame_gr_create.restype = C.c_int
_lib.flame_gr_forward.argtypes = [C.c_void_p, C.POINTER(flame_gr_weights), C.c_void_p, _i32p, C.c_void_p, _i32p,
                                  C.c_int32, C.c_void_p, C.c_void_p]
_lib.flame_gr_forward.restype = C.c_int
_lib.flame_gr_forward_hidden.argtypes = _lib.flame_gr_forward.argtypes
_lib.flame_gr_forward_hidden.restype = C.c_int
_lib.flame_gr_forward_static.argtypes = [C.POINTER(flame_gr_config), C.POINTER(flame_gr_weights), C.c_void_p, _i32p, C.c_void_p, _i32p,
                                         C.c_int32, C.c_void_p, C.c_void_p]
_lib.flame_gr_forward_static.restype = C.c_int
_lib.flame_gr_static_scratch_bytes.argtypes = [C.POINTER(flame_gr_config), C.c_int64, C.POINTER(C.c_int64)]
_lib.flame_gr_static_scratch_bytes.restype = C.c_int
_lib.flame_gr_capture.argtypes = [C.c_void_p, C.c_int32, C.POINTER(flame_gr_weights), C.c_void_p, _i32p, C.c_void_p, _i32p,
                                  C.c_int32, C.c_void_p, C.c_void_p]
_lib.flame_gr_capture.restype = C.c_int
_lib.flame_gr_replay.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
_lib.flame_gr_replay.restype = C.c_int
_lib.flame_gr_prefill.argtypes = [C.c_void_p, C.POINTER(flame_gr_weights), C.c_void_p, _i32p, _i32p, C.c_int32, C.c_void_p]
_lib.flame_gr_prefill.restype = C.c_int
_lib.flame_gr_score.argtypes = [C.c_void_p, C.POINTER(flame_gr_weights), C.c_void_p, _i32p, C.c_int32, C.c_void_p, C.c_void_p]
_lib.flame_gr_score.restype = C.c_int
_lib.flame_gr_destroy.argtypes = [C.c_void_p]
_lib.flame_gr_destroy.restype = C.c_int
_lib.flame_gr_last_error.argtypes = [C.c_void_p]
_lib.flame_gr_last_error.restype = C.c_char_p
_lib.flame_gr_host_bucket_table.argtypes = [C.c_int32, C.c_int32, _i32p]
_lib.flame_gr_host_bucket_table.restype = C.c_int
_lib.flame_gr_host_mask.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
_lib.flame_gr_host_mask.restype = C.c_int
_lib.flame_gr_host_plan.argtypes = [C.POINTER(flame_gr_config), _i32p, _i32p, C.c_int32, _i32p, _i32p, _i32p, C.c_int32]
_lib.flame_gr_host_plan.restype = C.c_int
_lib.flame_gr_host_workspace_rows.argtypes = [C.POINTER(flame_gr_config), C.POINTER(C.c_int64)]
_lib.flame_gr_host_workspace_rows.restype = C.c_int
_lib.flame_gr_host_plan_reserved.argtypes = [C.POINTER(flame_gr_config), _i32p, _i32p, _i32p, C.c_int32, _i32p, _i32p, C.c_int32]
_lib.flame_gr_host_plan_reserved.restype = C.c_int
_lib.flame_gr_debug_capture.argtypes = [C.c_void_p, C.c_int32]
_lib.flame_gr_debug_capture.restype = C.c_int
_lib.flame_gr_debug_stage.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
_lib.flame_gr_debug_stage.restype = C.c_int
_lib.flame_gr_debug_device_mask.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
_lib.flame_gr_debug_device_mask.restype = C.c_int
_lib.flame_gr_debug_profile.argtypes = [C.c_void_p, C.c_int32]
_lib.flame_gr_debug_profile.restype = C.c_int
_lib.flame_gr_debug_profile_read.argtypes = [C.c_void_p, C.POINTER(C.c_float), _i32p]
_lib.flame_gr_debug_profile_read.restype = C.c_int

class flame_dso_config(C.Structure):
    _fields_ = [("hist_len", C.c_int32), ("n_profiles", C.c_int32), ("profiles", _i32p),
                ("n_executors", C.c_int32), ("explicit_shapes", C.c_int32), ("max_batch", C.c_int32)]


_lib.flame_dso_create.argtypes = [C.POINTER(flame_gr_config), C.POINTER(flame_gr_weights), C.POINTER(flame_dso_config),
                                  C.POINTER(C.c_void_p)]
_lib.flame_dso_create.restype = C.c_int
_lib.flame_dso_submit.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.POINTER(C.c_int64)]
_lib.flame_dso_submit.restype = C.c_int
_lib.flame_dso_submit_jagged.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.POINTER(C.c_int64)]
_lib.flame_dso_submit_jagged.restype = C.c_int
_lib.flame_dso_wait.argtypes = [C.c_void_p, C.c_int64]
_lib.flame_dso_wait.restype = C.c_int
_lib.flame_dso_drain.argtypes = [C.c_void_p]
_lib.flame_dso_drain.restype = C.c_int
_lib.flame_dso_flush.argtypes = [C.c_void_p]
_lib.flame_dso_flush.restype = C.c_int
_lib.flame_dso_destroy.argtypes = [C.c_void_p]
_lib.flame_dso_destroy.restype = C.c_int
_lib.flame_dso_last_error.argtypes = [C.c_void_p]
_lib.flame_dso_last_error.restype = C.c_char_p
_lib.flame_dso_route.argtypes = [_i32p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, _i32p, C.c_int32, _i32p]
_lib.flame_dso_route.restype = C.c_int
_lib.flame_dso_stats.argtypes = [C.c_void_p, C.POINTER(C.c_int64)]
_lib.flame_dso_stats.restype = C.c_int

class flame_climber_head_config(C.Structure):
    _fields_ = [("n_blocks", C.c_int32), ("d_model", C.c_int32), ("n_tasks", C.c_int32), ("expert_width", C.c_int32)]


class flame_climber_head_weights(C.Structure):
    _fields_ = [("wg", C.c_void_p), ("cg", C.c_void_p), ("a_w", C.c_void_p), ("a_b", C.c_void_p), ("v", C.c_void_p),
                ("c", C.c_void_p)]


_lib.flame_climber_head.argtypes = [C.POINTER(flame_climber_head_config), C.POINTER(flame_climber_head_weights),
                                    C.POINTER(C.c_void_p), C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
_lib.flame_climber_head.restype = C.c_int
_lib.flame_climber_block_range.argtypes = [C.c_int32, C.c_int32, C.c_int32, _i32p, _i32p]
_lib.flame_climber_block_range.restype = C.c_int
_lib.flame_climber_last_error.argtypes = []
_lib.flame_climber_last_error.restype = C.c_char_p

CLIMBER_EXPORTS = ("flame_climber_head", "flame_climber_block_range", "flame_climber_last_error")

DSO_EXPORTS = ("flame_dso_create", "flame_dso_submit", "flame_dso_submit_jagged", "flame_dso_wait", "flame_dso_drain", "flame_dso_flush", "flame_dso_destroy",
               "flame_dso_last_error", "flame_dso_route", "flame_dso_stats")

EXPORTS = ("flame_gr_create", "flame_gr_forward", "flame_gr_forward_hidden", "flame_gr_forward_static", "flame_gr_static_scratch_bytes", "flame_gr_capture", "flame_gr_replay", "flame_gr_prefill", "flame_gr_score", "flame_gr_destroy",
           "flame_gr_last_error",
           "flame_gr_host_bucket_table", "flame_gr_host_mask", "flame_gr_host_plan", "flame_gr_host_plan_reserved", "flame_gr_host_workspace_rows",
           "flame_gr_debug_capture", "flame_gr_debug_stage", "flame_gr_debug_device_mask",
           "flame_gr_debug_profile", "flame_gr_debug_profile_read")


class FlameGRError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{STATUS.get(code, code)}: {msg}")
        self.code = code


def _check(rc: int, h=None):
    if rc != 0:
        msg = _lib.flame_gr_last_error(h)
        raise FlameGRError(rc, msg.decode() if msg else "")


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(t) -> Optional[int]:
    """Device (torch tensor) or host (numpy) pointer, or None."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr() if t.numel() else None


def make_config(n_layers, d_model, n_heads, n_buckets, max_rel_dist, dtype, *, ln_eps=1e-6, attn_scale=1.0,
                max_requests=0, max_total_tokens=0, max_seq_tokens=0, n_streams=0, kv_cache=0,
                attn_kind="silu", latency_mode=0, weights_static=0) -> flame_gr_config:
    dt = {"f32": FLAME_GR_F32, "bf16": FLAME_GR_BF16}.get(dtype, dtype)
    ak = {"silu": FLAME_GR_ATTN_SILU, "softmax": FLAME_GR_ATTN_SOFTMAX}.get(attn_kind, attn_kind)
    return flame_gr_config(n_layers, d_model, n_heads, n_buckets, max_rel_dist, dt, ln_eps, attn_scale,
                           max_requests, max_total_tokens, max_seq_tokens, n_streams, ak, int(kv_cache), int(latency_mode),
                           int(weights_static))


# ---------------------------------------------------------------------------------------------
# the three calls of the boundary, plus helpers, under their C names
# ---------------------------------------------------------------------------------------------
def flame_gr_create(cfg: flame_gr_config) -> C.c_void_p:
    h = C.c_void_p()
    _check(_lib.flame_gr_create(C.byref(cfg), C.byref(h)))
    return h


def flame_gr_destroy(h) -> None:
    _check(_lib.flame_gr_destroy(h))


def pack_weights(w: Dict[str, object]) -> flame_gr_weights:
    """dict of device tensors (+ python float b_s) -> struct of device pointers."""
    return flame_gr_weights(_ptr(w["w1"]), _ptr(w["b1"]), _ptr(w["rab"]), _ptr(w["ln_g"]), _ptr(w["ln_b"]),
                            _ptr(w["w2"]), _ptr(w["b2"]), _ptr(w.get("w_s")), float(w.get("b_s", 0.0)),
                            _ptr(w.get("temperature")))


def flame_gr_forward(h, weights, history_emb, history_offsets, cand_emb, cand_offsets, scores, stream=None) -> None:
    """weights: flame_gr_weights or dict; *_emb / scores: device tensors; *_offsets: host int32 arrays.
    stream: torch.cuda.Stream, raw hipStream_t integer, or None for the current torch stream."""
    ws = weights if isinstance(weights, flame_gr_weights) else pack_weights(weights)
    ho, co = _i32(history_offsets), _i32(cand_offsets)
    n = len(ho) - 1
    if len(co) - 1 != n:
        raise ValueError("offset arrays differ in length")
    if stream is None:
        sp = torch.cuda.current_stream().cuda_stream
    else:
        sp = getattr(stream, "cuda_stream", stream)
    rc = _lib.flame_gr_forward(h, C.byref(ws), _ptr(history_emb), ho.ctypes.data_as(_i32p), _ptr(cand_emb),
                               co.ctypes.data_as(_i32p), n, _ptr(scores), C.c_void_p(sp))
    _check(rc, h)


def flame_gr_forward_static(cfg: flame_gr_config, weights, history_emb, history_offsets, cand_emb, cand_offsets, scores,
                            stream=None) -> None:
    """flame_gr_forward without a handle, in the library's static device workspace (no allocation)."""
    ws = weights if isinstance(weights, flame_gr_weights) else pack_weights(weights)
    ho, co = _i32(history_offsets), _i32(cand_offsets)
    n = len(ho) - 1
    if len(co) - 1 != n:
        raise ValueError("offset arrays differ in length")
    sp = torch.cuda.current_stream().cuda_stream if stream is None else getattr(stream, "cuda_stream", stream)
    rc = _lib.flame_gr_forward_static(C.byref(cfg), C.byref(ws), _ptr(history_emb), ho.ctypes.data_as(_i32p), _ptr(cand_emb),
                                      co.ctypes.data_as(_i32p), n, _ptr(scores), C.c_void_p(sp))
    _check(rc)


def flame_gr_static_scratch_bytes(cfg: flame_gr_config, padded_rows: int) -> int:
    out = C.c_int64(0)
    _check(_lib.flame_gr_static_scratch_bytes(C.byref(cfg), padded_rows, C.byref(out)))
    return out.value


def _stream_ptr(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def flame_gr_capture(h, weights, history_emb, history_offsets, cand_emb, cand_offsets, scores, slot: int = 0,
                     record_stream=None) -> None:
    """Record the forward of this fixed batch (shape, buffers) into graph `slot` of the handle."""
    ws = weights if isinstance(weights, flame_gr_weights) else pack_weights(weights)
    ho, co = _i32(history_offsets), _i32(cand_offsets)
    n = len(ho) - 1
    if len(co) - 1 != n:
        raise ValueError("offset arrays differ in length")
    rc = _lib.flame_gr_capture(h, slot, C.byref(ws), _ptr(history_emb), ho.ctypes.data_as(_i32p), _ptr(cand_emb),
                               co.ctypes.data_as(_i32p), n, _ptr(scores),
                               C.c_void_p(getattr(record_stream, "cuda_stream", record_stream) or 0))
    _check(rc, h)


def flame_gr_replay(h, stream=None, slot: int = 0) -> None:
    _check(_lib.flame_gr_replay(h, slot, C.c_void_p(_stream_ptr(stream))), h)


def flame_gr_prefill(h, weights, history_emb, history_offsets, cand_capacity, stream=None) -> None:
    """History stage of the two-stage path; cand_capacity: host int32 [n_requests]."""
    ws = weights if isinstance(weights, flame_gr_weights) else pack_weights(weights)
    ho, cc = _i32(history_offsets), _i32(cand_capacity)
    n = len(ho) - 1
    if len(cc) != n:
        raise ValueError("cand_capacity must have one entry per request")
    rc = _lib.flame_gr_prefill(h, C.byref(ws), _ptr(history_emb), ho.ctypes.data_as(_i32p), cc.ctypes.data_as(_i32p), n,
                               C.c_void_p(_stream_ptr(stream)))
    _check(rc, h)


def flame_gr_score(h, weights, cand_emb, cand_offsets, scores, stream=None) -> None:
    """Candidate stage of the two-stage path, against the history cached by the last prefill."""
    ws = weights if isinstance(weights, flame_gr_weights) else pack_weights(weights)
    co = _i32(cand_offsets)
    rc = _lib.flame_gr_score(h, C.byref(ws), _ptr(cand_emb), co.ctypes.data_as(_i32p), len(co) - 1, _ptr(scores),
                             C.c_void_p(_stream_ptr(stream)))
    _check(rc, h)


def flame_gr_forward_hidden(h, weights, history_emb, history_offsets, cand_emb, cand_offsets, hidden, stream=None) -> None:
    """As flame_gr_forward, with the candidates' final residual rows (device fp32 [sum M, d]) as the output."""
    ws = weights if isinstance(weights, flame_gr_weights) else pack_weights(weights)
    ho, co = _i32(history_offsets), _i32(cand_offsets)
    n = len(ho) - 1
    if len(co) - 1 != n:
        raise ValueError("offset arrays differ in length")
    rc = _lib.flame_gr_forward_hidden(h, C.byref(ws), _ptr(history_emb), ho.ctypes.data_as(_i32p), _ptr(cand_emb),
                                      co.ctypes.data_as(_i32p), n, _ptr(hidden), C.c_void_p(_stream_ptr(stream)))
    _check(rc, h)


def flame_gr_last_error(h=None) -> str:
    return _lib.flame_gr_last_error(h).decode()


def flame_gr_host_bucket_table(n_buckets: int, max_rel_dist: int) -> np.ndarray:
    out = np.empty(max(max_rel_dist, 0), np.int32)
    _check(_lib.flame_gr_host_bucket_table(n_buckets, max_rel_dist, out.ctypes.data_as(_i32p)))
    return out


def flame_gr_host_mask(L: int, M: int, n_buckets: int, max_rel_dist: int):
    N = L + M
    mask = np.empty((N, N), np.uint8)
    bucket = np.empty((N, N), np.int32)
    _check(_lib.flame_gr_host_mask(L, M, n_buckets, max_rel_dist, mask.ctypes.data, bucket.ctypes.data))
    return mask, bucket


def flame_gr_host_plan(cfg: flame_gr_config, history_offsets, cand_offsets):
    """-> (tok_off [B+1], segments [S,6]: request, L, cand_begin, M, row_start, group)"""
    ho, co = _i32(history_offsets), _i32(cand_offsets)
    n = len(ho) - 1
    tok = np.zeros(n + 1, np.int32)
    nseg = C.c_int32(0)
    _check(_lib.flame_gr_host_plan(C.byref(cfg), ho.ctypes.data_as(_i32p), co.ctypes.data_as(_i32p), n,
                                   tok.ctypes.data_as(_i32p), C.byref(nseg), None, 0))
    seg = np.zeros((max(nseg.value, 1), 6), np.int32)
    _check(_lib.flame_gr_host_plan(C.byref(cfg), ho.ctypes.data_as(_i32p), co.ctypes.data_as(_i32p), n,
                                   tok.ctypes.data_as(_i32p), C.byref(nseg), seg.ctypes.data_as(_i32p), len(seg)))
    return tok, seg[:nseg.value]


def flame_gr_host_workspace_rows(cfg: flame_gr_config) -> int:
    rows = C.c_int64(0)
    _check(_lib.flame_gr_host_workspace_rows(C.byref(cfg), C.byref(rows)))
    return rows.value


def flame_gr_host_plan_reserved(cfg: flame_gr_config, history_offsets, cand_offsets, cand_capacity):
    """-> segments [S,6] of the two-stage layout: request, L, cand_begin, M, row_start, group"""
    ho, co, cc = _i32(history_offsets), _i32(cand_offsets), _i32(cand_capacity)
    n = len(ho) - 1
    if len(co) - 1 != n or len(cc) != n:
        raise ValueError("offset and capacity arrays differ in length")
    seg = np.zeros((max(n, 1), 6), np.int32)
    nseg = C.c_int32(0)
    _check(_lib.flame_gr_host_plan_reserved(C.byref(cfg), ho.ctypes.data_as(_i32p), co.ctypes.data_as(_i32p),
                                            cc.ctypes.data_as(_i32p), n, C.byref(nseg), seg.ctypes.data_as(_i32p), len(seg)))
    return seg[:nseg.value]


def flame_gr_debug_capture(h, layer: int) -> None:
    _check(_lib.flame_gr_debug_capture(h, layer), h)


def flame_gr_debug_stage(h, which: int, n_tokens: int, d: int) -> np.ndarray:
    out = np.empty((n_tokens, d), np.float32)
    _check(_lib.flame_gr_debug_stage(h, which, out.ctypes.data), h)
    return out


def flame_gr_debug_device_mask(h, L: int, M: int):
    N = L + M
    mask = np.empty((N, N), np.uint8)
    bucket = np.empty((N, N), np.int32)
    _check(_lib.flame_gr_debug_device_mask(h, L, M, mask.ctypes.data, bucket.ctypes.data), h)
    return mask, bucket


def flame_gr_debug_profile(h, enable: bool) -> None:
    _check(_lib.flame_gr_debug_profile(h, int(enable)), h)


def flame_gr_debug_profile_read(h):
    """-> {kind: (milliseconds, launches)} for the last forward run with profiling on."""
    ms = (C.c_float * len(KERNEL_KINDS))()
    n = (C.c_int32 * len(KERNEL_KINDS))()
    _check(_lib.flame_gr_debug_profile_read(h, ms, n), h)
    return {k: (float(ms[i]), int(n[i])) for i, k in enumerate(KERNEL_KINDS)}


# ---------------------------------------------------------------------------------------------
# request orchestrator (include/flame_dso.h); embeddings and scores are HOST numpy arrays here
# ---------------------------------------------------------------------------------------------
def _dso_check(rc: int, dso=None):
    if rc != 0:
        msg = _lib.flame_dso_last_error(dso)
        raise FlameGRError(rc, msg.decode() if msg else "")


def flame_dso_create(cfg: flame_gr_config, weights, hist_len: int, profiles, n_executors: int,
                     explicit_shapes=True, max_batch: int = 1) -> C.c_void_p:
    """explicit_shapes: True/1 graph executors, False/0 eager dynamic shapes, 2 jagged micro-batches of max_batch."""
    ws = weights if isinstance(weights, flame_gr_weights) else pack_weights(weights)
    prof = _i32(profiles)
    dc = flame_dso_config(hist_len, len(prof), prof.ctypes.data_as(_i32p), n_executors, int(explicit_shapes), max_batch)
    out = C.c_void_p()
    _dso_check(_lib.flame_dso_create(C.byref(cfg), C.byref(ws), C.byref(dc), C.byref(out)))
    return out


def host_embedding(a, dtype: str) -> np.ndarray:
    """fp32 numpy values -> the raw host layout the orchestrator expects (bf16 as uint16 bit patterns;
    the values are expected to be bf16-representable already, as the workload generators make them)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return a
    bits = a.view(np.uint32)
    if (bits & 0xFFFF).any():
        raise ValueError("values are not bf16-representable")
    return np.ascontiguousarray((bits >> 16).astype(np.uint16))


def flame_dso_submit(dso, history_emb: np.ndarray, cand_emb: np.ndarray, scores: np.ndarray) -> int:
    """history_emb / cand_emb: contiguous host arrays in the model dtype (see host_embedding);
    scores: contiguous float32 host array [n_cand], filled by the wait that retires the ticket."""
    if not (cand_emb.flags.c_contiguous and scores.flags.c_contiguous and scores.dtype == np.float32):
        raise ValueError("cand_emb and scores must be contiguous, scores float32")
    t = C.c_int64(0)
    hp = history_emb.ctypes.data if history_emb is not None and history_emb.size else None
    _dso_check(_lib.flame_dso_submit(dso, hp, cand_emb.ctypes.data, int(cand_emb.shape[0]), scores.ctypes.data, C.byref(t)), dso)
    return t.value


def flame_dso_submit_jagged(dso, history_emb: np.ndarray, cand_emb: np.ndarray, scores: np.ndarray) -> int:
    """Mode 2: a request whose history length is history_emb.shape[0] (at most the capacity given at create)."""
    if not (cand_emb.flags.c_contiguous and scores.flags.c_contiguous and scores.dtype == np.float32):
        raise ValueError("cand_emb and scores must be contiguous, scores float32")
    L = int(history_emb.shape[0]) if history_emb is not None else 0
    if L and not history_emb.flags.c_contiguous:
        raise ValueError("history_emb must be contiguous")
    t = C.c_int64(0)
    hp = history_emb.ctypes.data if L else None
    _dso_check(_lib.flame_dso_submit_jagged(dso, hp, L, cand_emb.ctypes.data, int(cand_emb.shape[0]), scores.ctypes.data,
                                            C.byref(t)), dso)
    return t.value


def flame_dso_wait(dso, ticket: int) -> None:
    _dso_check(_lib.flame_dso_wait(dso, ticket), dso)


def flame_dso_flush(dso) -> None:
    _dso_check(_lib.flame_dso_flush(dso), dso)


def flame_dso_drain(dso) -> None:
    _dso_check(_lib.flame_dso_drain(dso), dso)


def flame_dso_destroy(dso) -> None:
    _dso_check(_lib.flame_dso_destroy(dso))


def flame_dso_last_error(dso=None) -> str:
    return _lib.flame_dso_last_error(dso).decode()


def flame_dso_stats(dso) -> Dict[str, int]:
    out = (C.c_int64 * 4)()
    _dso_check(_lib.flame_dso_stats(dso, out), dso)
    return dict(zip(("requests", "chunks", "candidate_rows_computed", "waits_for_a_busy_executor"), (int(v) for v in out)))


def flame_dso_route(profiles, hist_len: int, d_model: int, n_cand: int, explicit_shapes: bool = True):
    """-> list of (profile index, candidates taken)"""
    prof = _i32(profiles)
    n = C.c_int32(0)
    rc = _lib.flame_dso_route(prof.ctypes.data_as(_i32p), len(prof), hist_len, d_model, int(explicit_shapes), n_cand, None, 0,
                              C.byref(n))
    if rc not in (0, -2):
        raise FlameGRError(rc, "flame_dso_route")
    buf = np.zeros((max(n.value, 1), 2), np.int32)
    rc = _lib.flame_dso_route(prof.ctypes.data_as(_i32p), len(prof), hist_len, d_model, int(explicit_shapes), n_cand,
                              buf.ctypes.data_as(_i32p), len(buf), C.byref(n))
    if rc != 0:
        raise FlameGRError(rc, "flame_dso_route")
    return [(int(a), int(b)) for a, b in buf[:n.value]]


# ---------------------------------------------------------------------------------------------
# fusion of the sub-sequence blocks and task head (include/flame_climber.h)
# ---------------------------------------------------------------------------------------------
def flame_climber_block_range(L: int, n_blocks: int, b: int):
    lo, hi = C.c_int32(0), C.c_int32(0)
    rc = _lib.flame_climber_block_range(L, n_blocks, b, C.byref(lo), C.byref(hi))
    if rc != 0:
        raise FlameGRError(rc, "flame_climber_block_range")
    return lo.value, hi.value


def flame_climber_head(head: Dict[str, object], hidden, fused, probs, stream=None) -> None:
    """head: dict of device fp32 tensors wg [Nb,d,Nb*d], cg [Nb,d], a_w [T,E,d], a_b [T,E], v [T,E], c [T];
    hidden: list of Nb device fp32 tensors [rows, d]; fused [rows, d] workspace; probs [rows, T] output."""
    nb = len(hidden)
    rows, d = (int(hidden[0].shape[0]), int(hidden[0].shape[1])) if nb else (0, 0)
    T, E = int(head["a_w"].shape[0]), int(head["a_w"].shape[1])
    cfg = flame_climber_head_config(nb, d, T, E)
    ws = flame_climber_head_weights(*[_ptr(head[k]) for k in ("wg", "cg", "a_w", "a_b", "v", "c")])
    ptrs = (C.c_void_p * max(nb, 1))(*[_ptr(h) for h in hidden])
    rc = _lib.flame_climber_head(C.byref(cfg), C.byref(ws), ptrs, rows, _ptr(fused), _ptr(probs), C.c_void_p(_stream_ptr(stream)))
    if rc != 0:
        raise FlameGRError(rc, _lib.flame_climber_last_error().decode())


# ---------------------------------------------------------------------------------------------
# marshalling of a numpy workload into device tensors
# ---------------------------------------------------------------------------------------------
def to_device(workload, device="cuda:0"):
    """Upload a workloads.Workload: returns (cfg struct fields dict, weights dict, hist, cand) as
    torch tensors of the workload's storage dtype (bf16 values are already exactly representable)."""
    dt = torch.bfloat16 if workload.cfg.dtype == "bf16" else torch.float32

    def up(a, dtype=dt):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device=device, dtype=dtype)

    w = workload.weights
    dw = {k: up(w[k]) for k in ("w1", "b1", "ln_g", "ln_b", "w2", "b2", "w_s")}
    dw["rab"] = up(w["rab"], torch.float32)
    dw["b_s"] = float(w["b_s"])
    if "temperature" in w:
        dw["temperature"] = up(w["temperature"], torch.float32)
    return dw, up(workload.history_emb), up(workload.cand_emb)


def config_for(workload, *, n_streams=0, max_seq_tokens=0, slack_requests=0, kv_cache=0, slack_tokens=0,
               latency_mode=0, weights_static=0) -> flame_gr_config:
    c = workload.cfg
    tot = int(workload.history_offsets[-1]) + int(workload.cand_offsets[-1])
    return make_config(c.n_layers, c.d_model, c.n_heads, c.n_buckets, c.max_rel_dist, c.dtype,
                       ln_eps=c.ln_eps, attn_scale=c.attn_scale,
                       max_requests=workload.n_requests + slack_requests, max_total_tokens=tot + slack_tokens,
                       max_seq_tokens=max_seq_tokens, n_streams=n_streams, kv_cache=kv_cache,
                       attn_kind=getattr(c, "attn_kind", "silu"), latency_mode=latency_mode, weights_static=weights_static)
