"""ctypes binding of libcachefocus.so: one Python function per C entry point, same names.

Argument marshalling only: tensors are torch CUDA tensors (PyTorch is used for device
memory and streams, nothing else), pointers are taken with ``data_ptr()``, the current
torch stream is passed unless one is given.  There is no fallback: if the shared library
has not been built, loading raises.
"""

from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcachefocus.so")

CF_OK, CF_ERR_INVALID_ARG, CF_ERR_UNSUPPORTED, CF_ERR_RANGE, CF_ERR_WORKSPACE, CF_ERR_DEVICE = 0, -1, -2, -3, -4, -5
CF_F32, CF_BF16, CF_F16 = 0, 1, 2
CF_ROPE_HALF, CF_ROPE_INTERLEAVED = 0, 1
CF_SEG_PREFIX, CF_SEG_DOC, CF_SEG_SELF = 0, 1, 2
CF_ALLOC_KEEP, CF_ALLOC_ALIGN, CF_ALLOC_SORT = 0, 1, 2
CF_FLAG_BAD_SEGMENT, CF_FLAG_NONFINITE_SCORE, CF_FLAG_DOC_TOO_LONG, CF_FLAG_POS_OVERFLOW, CF_FLAG_BAD_INDEX = 1, 2, 4, 8, 16
CF_FLAG_POS_RANGE = 32

DTYPE_CODE = {"f32": CF_F32, "bf16": CF_BF16, "f16": CF_F16}

EXPORTS = ("cf_reposition_keys", "cf_prefill_workspace_bytes", "cf_prefill_attention", "cf_prune_topk",
           "cf_assign_positions", "cf_gather_segments", "cf_last_error", "cf_version", "cf_calibrate", "cf_profile_kernel_events", "cf_profile_kernel_ms",
           "cf_prefill_layer", "cf_assemble_cache", "cf_prefill_attention_static")
CF_STATIC_SCRATCH_BYTES = 32 << 20
CF_MAX_PENDING = 15


class cf_layer_desc(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("dtype", C.c_int32), ("rope_pairing", C.c_int32), ("max_positions", C.c_int32),
                ("rope_base", C.c_double), ("softmax_scale", C.c_float), ("reserved", C.c_int32),
                ("store_token_stride", C.c_int64), ("store_head_stride", C.c_int64)]


class cf_prune_step(C.Structure):
    _fields_ = [("keep", C.c_int32), ("strategy", C.c_int32), ("force_n_reuse", C.c_int32),
                ("normalise_by_len", C.c_int32), ("stride", C.c_int32), ("pos_begin", C.c_int32),
                ("pos_end", C.c_int32), ("prefix_len", C.c_int32), ("doc_stored_start", C.c_int32),
                ("reserved", C.c_int32),
                ("doc_tok_offset", C.c_void_p), ("doc_len", C.c_void_p), ("cand", C.c_void_p), ("n_cand", C.c_void_p),
                ("keep_idx", C.c_void_p), ("n_keep", C.c_void_p), ("new_start", C.c_void_p), ("q_start", C.c_void_p),
                ("n_reuse", C.c_void_p), ("order", C.c_void_p), ("next_segs", C.c_void_p), ("next_n_seg", C.c_void_p)]


SEGMENT_DTYPE = np.dtype([("tok_offset", "<i8"), ("len", "<i4"), ("stored_start", "<i4"),
                          ("new_start", "<i4"), ("kind", "<i4"), ("doc", "<i4"), ("reserved", "<i4")])
assert SEGMENT_DTYPE.itemsize == 32


class CacheFocusError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"cf_status {status}: {message}")
        self.status = status
        self.message = message


_lib = None


def load() -> C.CDLL:
    """Load libcachefocus.so (built by paper_2502_11101_amd.build); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} not found: build it with `python -m paper_2502_11101_amd.build`")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    dp = C.POINTER(cf_layer_desc)
    lib.cf_last_error.restype = C.c_char_p
    lib.cf_last_error.argtypes = []
    lib.cf_version.restype = i32
    lib.cf_version.argtypes = []
    lib.cf_calibrate.restype = i32
    lib.cf_calibrate.argtypes = [i32, vp, vp, sz, i32, i32, vp, C.POINTER(C.c_double), vp]
    lib.cf_profile_kernel_events.restype = i32
    lib.cf_profile_kernel_events.argtypes = [i32]
    lib.cf_profile_kernel_ms.restype = i32
    lib.cf_profile_kernel_ms.argtypes = [C.POINTER(C.c_double), C.POINTER(i32)]
    lib.cf_reposition_keys.restype = i32
    lib.cf_reposition_keys.argtypes = [dp, vp, vp, vp, i32, i64, i32, vp, vp]
    lib.cf_prefill_workspace_bytes.restype = sz
    lib.cf_prefill_workspace_bytes.argtypes = [dp, i32, i32, i32, i64]
    lib.cf_prefill_attention.restype = i32
    lib.cf_prefill_attention.argtypes = [dp, vp, vp, i32, vp, vp, vp, i64, vp, vp, vp, vp, i32, i32, i32, i64,
                                         vp, vp, vp, i32, vp, sz, vp, vp]
    lib.cf_prefill_attention_static.restype = i32
    lib.cf_prefill_attention_static.argtypes = [dp, vp, vp, i32, vp, vp, vp, i64, vp, vp, vp, vp, i32, i32, i32, i64,
                                                vp, vp, vp, i32, vp, vp]
    lib.cf_prefill_layer.restype = i32
    lib.cf_prefill_layer.argtypes = [dp, vp, vp, i32, vp, vp, vp, i64, vp, vp, vp, vp, i32, i32, i32, i64,
                                     vp, vp, vp, i32, vp, sz, C.POINTER(cf_prune_step), i32, i32, vp, vp]
    lib.cf_prune_topk.restype = i32
    lib.cf_prune_topk.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp]
    lib.cf_assign_positions.restype = i32
    lib.cf_assign_positions.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.cf_assemble_cache.restype = i32
    lib.cf_assemble_cache.argtypes = [dp, vp, vp, i64, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, i64, i64, i64, vp, vp, vp,
                                      vp, vp, vp]
    lib.cf_gather_segments.restype = i32
    lib.cf_gather_segments.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, i32, vp, vp]
    _lib = lib
    return lib


def make_desc(n_q_heads: int, n_kv_heads: int, head_dim: int, dtype, rope_base: float, max_positions: int,
              rope_pairing: int = CF_ROPE_HALF, softmax_scale: float = 0.0, store_token_stride: int = 0,
              store_head_stride: int = 0) -> cf_layer_desc:
    """Strides (elements) describe the cache store; 0, 0 is token-major [token][kv head][head_dim]."""
    code = DTYPE_CODE[dtype] if isinstance(dtype, str) else int(dtype)
    return cf_layer_desc(n_q_heads, n_kv_heads, head_dim, code, rope_pairing, max_positions, float(rope_base),
                         float(softmax_scale), 0, int(store_token_stride), int(store_head_stride))


def segments_array(segments: Sequence) -> np.ndarray:
    """Pack (tok_offset, len, stored_start, new_start, kind, doc) tuples into the 32-byte table layout."""
    arr = np.zeros(len(segments), dtype=SEGMENT_DTYPE)
    for i, s in enumerate(segments):
        arr[i] = (s[0], s[1], s[2], s[3], s[4], s[5] if len(s) > 5 else -1, 0)
    return arr


def segments_to_device(arr: np.ndarray, device="cuda"):
    import torch
    raw = np.ascontiguousarray(arr).view(np.uint8).reshape(-1)
    if raw.size == 0:
        return torch.zeros(32, dtype=torch.uint8, device=device)
    return torch.from_numpy(raw.copy()).to(device)


def segments_from_device(t, count: int) -> np.ndarray:
    raw = t.detach().cpu().numpy().view(np.uint8).reshape(-1)[:count * 32]
    return raw.view(SEGMENT_DTYPE).copy()


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _check(status: int) -> None:
    if status != CF_OK:
        raise CacheFocusError(status, load().cf_last_error().decode())


def cf_version() -> int:
    return load().cf_version()


CF_CALIB_READ, CF_CALIB_COPY, CF_CALIB_MFMA_BF16, CF_CALIB_MFMA_F16 = 0, 1, 2, 3


def cf_calibrate(kind: int, src, dst, nbytes: int, workgroups: int, iters: int, sink, stream=None) -> float:
    """Enqueues one calibration kernel; returns the launch's flop count (0 for the memory kinds)."""
    flops = C.c_double(0.0)
    _check(load().cf_calibrate(kind, _ptr(src), _ptr(dst), nbytes, workgroups, iters, _ptr(sink), C.byref(flops),
                               _stream(stream)))
    return flops.value


def cf_profile_kernel_events(enable: bool) -> None:
    _check(load().cf_profile_kernel_events(1 if enable else 0))


def cf_profile_kernel_ms():
    """(mean milliseconds, launches) of the attention kernel's bracketed launches."""
    mean, n = C.c_double(0.0), C.c_int32(0)
    _check(load().cf_profile_kernel_ms(C.byref(mean), C.byref(n)))
    return mean.value, n.value


def cf_last_error() -> str:
    return load().cf_last_error().decode()


def cf_reposition_keys(desc, k_in, k_out, segs, n_seg: int, n_store_tokens: int, max_seg_len: int,
                       dev_flag=None, stream=None) -> None:
    _check(load().cf_reposition_keys(C.byref(desc), _ptr(k_in), _ptr(k_out), _ptr(segs), n_seg, n_store_tokens,
                                     max_seg_len, _ptr(dev_flag), _stream(stream)))


def cf_prefill_workspace_bytes(desc, batch: int, max_tq: int, seg_stride: int, max_kv_tokens: int) -> int:
    return int(load().cf_prefill_workspace_bytes(C.byref(desc), batch, max_tq, seg_stride, max_kv_tokens))


def cf_prefill_attention(desc, q, q_off, q_stored_start: int, q_new_start, k_store, v_store, n_store_tokens: int,
                         k_self, v_self, segs, n_seg, seg_stride: int, batch: int, max_tq: int,
                         max_kv_tokens: int, out, mass, score_accum, score_stride: int, workspace,
                         workspace_bytes: int, dev_flag=None, stream=None) -> None:
    _check(load().cf_prefill_attention(
        C.byref(desc), _ptr(q), _ptr(q_off), q_stored_start, _ptr(q_new_start), _ptr(k_store), _ptr(v_store),
        n_store_tokens, _ptr(k_self), _ptr(v_self), _ptr(segs), _ptr(n_seg), seg_stride, batch, max_tq,
        max_kv_tokens, _ptr(out), _ptr(mass), _ptr(score_accum), score_stride, _ptr(workspace), workspace_bytes,
        _ptr(dev_flag), _stream(stream)))


def cf_prefill_attention_static(desc, q, q_off, q_stored_start: int, q_new_start, k_store, v_store, n_store_tokens: int,
                                k_self, v_self, segs, n_seg, seg_stride: int, batch: int, max_tq: int,
                                max_kv_tokens: int, out, mass, score_accum, score_stride: int, dev_flag=None,
                                stream=None) -> None:
    _check(load().cf_prefill_attention_static(
        C.byref(desc), _ptr(q), _ptr(q_off), q_stored_start, _ptr(q_new_start), _ptr(k_store), _ptr(v_store),
        n_store_tokens, _ptr(k_self), _ptr(v_self), _ptr(segs), _ptr(n_seg), seg_stride, batch, max_tq,
        max_kv_tokens, _ptr(out), _ptr(mass), _ptr(score_accum), score_stride, _ptr(dev_flag), _stream(stream)))


def make_prune_step(keep: int, strategy: int, force_n_reuse: int, normalise_by_len: bool, stride: int, pos_begin: int,
                    pos_end: int, prefix_len: int, doc_stored_start: int, doc_tok_offset, doc_len, cand, n_cand,
                    keep_idx, n_keep, new_start, q_start, n_reuse, order, next_segs, next_n_seg) -> cf_prune_step:
    return cf_prune_step(keep, strategy, force_n_reuse, 1 if normalise_by_len else 0, stride, pos_begin, pos_end,
                         prefix_len, doc_stored_start, 0, _ptr(doc_tok_offset), _ptr(doc_len), _ptr(cand), _ptr(n_cand),
                         _ptr(keep_idx), _ptr(n_keep), _ptr(new_start), _ptr(q_start), _ptr(n_reuse), _ptr(order),
                         _ptr(next_segs), _ptr(next_n_seg))


def cf_prefill_layer(desc, q, q_off, q_stored_start: int, q_new_start, k_store, v_store, n_store_tokens: int,
                     k_self, v_self, segs, n_seg, seg_stride: int, batch: int, max_tq: int, max_kv_tokens: int, out,
                     mass, score_accum, score_stride: int, workspace, workspace_bytes: int,
                     prune: Optional[cf_prune_step] = None, dev_flag=None, stream=None, n_pending: int = 0,
                     defer: bool = False) -> None:
    _check(load().cf_prefill_layer(
        C.byref(desc), _ptr(q), _ptr(q_off), q_stored_start, _ptr(q_new_start), _ptr(k_store), _ptr(v_store),
        n_store_tokens, _ptr(k_self), _ptr(v_self), _ptr(segs), _ptr(n_seg), seg_stride, batch, max_tq,
        max_kv_tokens, _ptr(out), _ptr(mass), _ptr(score_accum), score_stride, _ptr(workspace), workspace_bytes,
        C.byref(prune) if prune is not None else None, n_pending, 1 if defer else 0, _ptr(dev_flag), _stream(stream)))


def cf_assemble_cache(desc, k_store, v_store, n_store_tokens: int, k_self, v_self, q_off, segs, n_seg, seg_stride: int,
                      batch: int, max_tq: int, max_seg_len: int, final_off, final_capacity: int, final_token_stride: int,
                      final_head_stride: int, k_final, v_final, final_len, final_pos=None, dev_flag=None,
                      stream=None) -> None:
    _check(load().cf_assemble_cache(
        C.byref(desc), _ptr(k_store), _ptr(v_store), n_store_tokens, _ptr(k_self), _ptr(v_self), _ptr(q_off), _ptr(segs),
        _ptr(n_seg), seg_stride, batch, max_tq, max_seg_len, _ptr(final_off), final_capacity, final_token_stride,
        final_head_stride, _ptr(k_final), _ptr(v_final), _ptr(final_len), _ptr(final_pos), _ptr(dev_flag), _stream(stream)))


def cf_prune_topk(score, len_, cand, n_cand, keep: int, batch: int, stride: int, keep_idx, n_keep,
                  dev_flag=None, stream=None) -> None:
    _check(load().cf_prune_topk(_ptr(score), _ptr(len_), _ptr(cand), _ptr(n_cand), keep, batch, stride,
                                _ptr(keep_idx), _ptr(n_keep), _ptr(dev_flag), _stream(stream)))


def cf_assign_positions(len_, ranked, n_ranked, batch: int, stride: int, pos_begin: int, pos_end: int,
                        strategy: int, force_n_reuse: int, new_start, q_start, n_reuse, order,
                        dev_flag=None, stream=None) -> None:
    _check(load().cf_assign_positions(_ptr(len_), _ptr(ranked), _ptr(n_ranked), batch, stride, pos_begin, pos_end,
                                      strategy, force_n_reuse, _ptr(new_start), _ptr(q_start), _ptr(n_reuse),
                                      _ptr(order), _ptr(dev_flag), _stream(stream)))


def cf_gather_segments(doc_tok_offset, len_, order, n_order, new_start, q_start, q_off, batch: int, stride: int,
                       prefix_len: int, doc_stored_start: int, q_stored_start: int, segs, n_seg, seg_stride: int,
                       dev_flag=None, stream=None) -> None:
    _check(load().cf_gather_segments(_ptr(doc_tok_offset), _ptr(len_), _ptr(order), _ptr(n_order), _ptr(new_start),
                                     _ptr(q_start), _ptr(q_off), batch, stride, prefix_len, doc_stored_start,
                                     q_stored_start, _ptr(segs), _ptr(n_seg), seg_stride, _ptr(dev_flag),
                                     _stream(stream)))
