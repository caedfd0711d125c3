"""ctypes binding of libsdllm.so: argument marshalling only.

Every function here has the name and argument order of its C counterpart in include/sdllm.h and
does nothing but turn torch tensors into device pointers / strides and status codes into
exceptions.  All arithmetic runs in the HIP kernels.  There is no fallback: if the shared library
has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsdllm.so")

# constants of include/sdllm.h
SDLLM_OK = 0
SDLLM_ERR_INVALID_ARG, SDLLM_ERR_UNSUPPORTED, SDLLM_ERR_WORKSPACE, SDLLM_ERR_HIP, SDLLM_ERR_STATIC_LIMIT = -1, -2, -3, -4, -5
SDLLM_STATIC_SCRATCH_BYTES = 8 << 20
SDLLM_BF16, SDLLM_F32 = 0, 1
SDLLM_SOFTMAX_MEAN, SDLLM_LOGIT_MEAN = 0, 1
SDLLM_PER_SEGMENT, SDLLM_JOINT = 0, 1
SDLLM_CEIL, SDLLM_FLOOR = 0, 1
SDLLM_MAX_POOL, SDLLM_AVG_POOL = 0, 1
SDLLM_EVICT_BIDIRECTIONAL, SDLLM_EVICT_PREFIX_ONLY = 0, 1
SDLLM_STATE_FULL, SDLLM_STATE_UPDATE, SDLLM_STATE_REUSE = 0, 1, 2
SDLLM_OP_SCORE_SELECT, SDLLM_OP_COMPACT_KV, SDLLM_OP_SPARSE_ATTN, SDLLM_OP_BLOCK_STEP = 0, 1, 2, 3

EXPORTED = ("sdllm_error_string", "sdllm_version", "sdllm_retained_count", "sdllm_workspace_bytes",
            "sdllm_cache_state", "sdllm_score_select", "sdllm_compact_kv", "sdllm_sparse_attn",
            "sdllm_sparse_attn_noalloc", "sdllm_block_step", "sdllm_dense_attn", "sdllm_stream_read_probe")


class sdllm_shape_t(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("seq_len", ctypes.c_int32), ("block_off", ctypes.c_int32),
        ("block_len", ctypes.c_int32), ("dtype", ctypes.c_int32), ("pool_kernel", ctypes.c_int32),
        ("score_mode", ctypes.c_int32), ("select_mode", ctypes.c_int32), ("k_rounding", ctypes.c_int32),
        ("pool_mode", ctypes.c_int32), ("evict_scope", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
        ("reserved", ctypes.c_int32), ("retention", ctypes.c_double),
        ("q_stride", ctypes.c_int64 * 3), ("kv_stride", ctypes.c_int64 * 3), ("blk_stride", ctypes.c_int64 * 3),
        ("cache_stride", ctypes.c_int64 * 3), ("out_stride", ctypes.c_int64 * 3),
    ]


class SdllmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({error_string(status)})")


_lib = None


def load() -> ctypes.CDLL:
    """Load libsdllm.so (once).  Raises if it has not been built: there is no other code path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2508_02558_amd.build` "
                           "(the HIP library is the only implementation; there is no fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    shp = ctypes.POINTER(sdllm_shape_t)
    i32p = ctypes.POINTER(ctypes.c_int32)
    lib.sdllm_error_string.restype = ctypes.c_char_p
    lib.sdllm_error_string.argtypes = [i32]
    lib.sdllm_version.restype = i32
    lib.sdllm_version.argtypes = []
    lib.sdllm_retained_count.restype = i32
    lib.sdllm_retained_count.argtypes = [shp, i32p, i32p, i32p]
    lib.sdllm_workspace_bytes.restype = i32
    lib.sdllm_workspace_bytes.argtypes = [shp, i32, i32, ctypes.POINTER(sz)]
    lib.sdllm_cache_state.restype = i32
    lib.sdllm_cache_state.argtypes = [i32, i32, i32p]
    lib.sdllm_score_select.restype = i32
    lib.sdllm_score_select.argtypes = [shp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.sdllm_compact_kv.restype = i32
    lib.sdllm_compact_kv.argtypes = [shp, vp, vp, vp, vp, vp, vp]
    lib.sdllm_sparse_attn.restype = i32
    lib.sdllm_sparse_attn.argtypes = [shp, vp, vp, vp, i32, vp, vp, vp, vp, sz, vp]
    lib.sdllm_sparse_attn_noalloc.restype = i32
    lib.sdllm_sparse_attn_noalloc.argtypes = [shp, vp, vp, vp, i32, vp, vp, vp, vp]
    lib.sdllm_block_step.restype = i32
    lib.sdllm_block_step.argtypes = [shp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, i32p]
    lib.sdllm_dense_attn.restype = i32
    lib.sdllm_dense_attn.argtypes = [shp, vp, ctypes.POINTER(ctypes.c_int64), vp, vp, vp, ctypes.POINTER(ctypes.c_int64), vp]
    lib.sdllm_stream_read_probe.restype = i32
    lib.sdllm_stream_read_probe.argtypes = [vp, sz, vp, vp]
    _lib = lib
    return lib


def error_string(status: int) -> str:
    return load().sdllm_error_string(status).decode()


def _check(status: int, where: str) -> None:
    if status != SDLLM_OK:
        raise SdllmError(status, where)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def strides_of(t) -> Tuple[int, int, int]:
    """{batch, head, row} element strides of a [B, H, n, d] tensor whose last axis is contiguous."""
    assert t.dim() == 4 and (t.shape[3] == 1 or t.stride(3) == 1), "last axis must be contiguous"
    return (t.stride(0), t.stride(1), t.stride(2))


def make_shape(*, batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int, seq_len: int, block_off: int,
               block_len: int, dtype: int, retention: float = 0.5, pool_kernel: int = 3,
               score_mode: int = SDLLM_SOFTMAX_MEAN, select_mode: int = SDLLM_PER_SEGMENT,
               k_rounding: int = SDLLM_CEIL, pool_mode: int = SDLLM_MAX_POOL,
               evict_scope: int = SDLLM_EVICT_BIDIRECTIONAL, softmax_scale: float = 0.0,
               q_stride: Optional[Sequence[int]] = None, kv_stride: Optional[Sequence[int]] = None,
               blk_stride: Optional[Sequence[int]] = None, cache_stride: Optional[Sequence[int]] = None,
               out_stride: Optional[Sequence[int]] = None, cache_rows: Optional[int] = None) -> sdllm_shape_t:
    """Fill an sdllm_shape_t; strides left out default to dense [B, H, n, d] tensors."""
    s = sdllm_shape_t()
    s.batch, s.n_q_heads, s.n_kv_heads, s.head_dim = batch, n_q_heads, n_kv_heads, head_dim
    s.seq_len, s.block_off, s.block_len, s.dtype = seq_len, block_off, block_len, dtype
    s.pool_kernel, s.score_mode, s.select_mode, s.k_rounding = pool_kernel, score_mode, select_mode, k_rounding
    s.pool_mode, s.evict_scope, s.softmax_scale, s.reserved = pool_mode, evict_scope, softmax_scale, 0
    s.retention = retention

    def dense(heads, rows):
        return (heads * rows * head_dim, rows * head_dim, head_dim)

    if cache_rows is None:
        cache_rows = max(1, seq_len - block_len)
    for name, val, dflt in (("q_stride", q_stride, dense(n_q_heads, block_len)),
                            ("kv_stride", kv_stride, dense(n_kv_heads, seq_len)),
                            ("blk_stride", blk_stride, dense(n_kv_heads, block_len)),
                            ("cache_stride", cache_stride, dense(n_kv_heads, cache_rows)),
                            ("out_stride", out_stride, dense(n_q_heads, block_len))):
        v = tuple(val) if val is not None else dflt
        setattr(s, name, (ctypes.c_int64 * 3)(*v))
    return s


# ------------------------------------------------------------------ the C entry points
def sdllm_version() -> int:
    return load().sdllm_version()


def sdllm_retained_count(shape: sdllm_shape_t) -> Tuple[int, int, int]:
    kt, kp, ks = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    _check(load().sdllm_retained_count(ctypes.byref(shape), ctypes.byref(kt), ctypes.byref(kp), ctypes.byref(ks)),
           "sdllm_retained_count")
    return kt.value, kp.value, ks.value


def sdllm_workspace_bytes(shape: sdllm_shape_t, op: int, n_cached: int = 0) -> int:
    out = ctypes.c_size_t()
    _check(load().sdllm_workspace_bytes(ctypes.byref(shape), op, n_cached, ctypes.byref(out)), "sdllm_workspace_bytes")
    return out.value


def sdllm_cache_state(step_in_block: int, delay: int = 1) -> int:
    st = ctypes.c_int32()
    _check(load().sdllm_cache_state(step_in_block, delay, ctypes.byref(st)), "sdllm_cache_state")
    return st.value


def sdllm_score_select(shape, q_blk, k_full, idx_out, pooled_out, score_out, ws, stream=None) -> None:
    _check(load().sdllm_score_select(ctypes.byref(shape), _ptr(q_blk), _ptr(k_full), _ptr(idx_out), _ptr(pooled_out),
                                     _ptr(score_out), _ptr(ws), ws.numel() * ws.element_size() if ws is not None else 0,
                                     _stream(stream)), "sdllm_score_select")


def sdllm_compact_kv(shape, k_full, v_full, idx, k_cache, v_cache, stream=None) -> None:
    _check(load().sdllm_compact_kv(ctypes.byref(shape), _ptr(k_full), _ptr(v_full), _ptr(idx), _ptr(k_cache),
                                   _ptr(v_cache), _stream(stream)), "sdllm_compact_kv")


def sdllm_sparse_attn(shape, q_blk, k_cache, v_cache, n_cached, k_blk, v_blk, out, ws, stream=None) -> None:
    _check(load().sdllm_sparse_attn(ctypes.byref(shape), _ptr(q_blk), _ptr(k_cache), _ptr(v_cache), n_cached,
                                    _ptr(k_blk), _ptr(v_blk), _ptr(out), _ptr(ws),
                                    ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream)),
           "sdllm_sparse_attn")


def sdllm_sparse_attn_noalloc(shape, q_blk, k_cache, v_cache, n_cached, k_blk, v_blk, out, stream=None) -> None:
    _check(load().sdllm_sparse_attn_noalloc(ctypes.byref(shape), _ptr(q_blk), _ptr(k_cache), _ptr(v_cache), n_cached,
                                            _ptr(k_blk), _ptr(v_blk), _ptr(out), _stream(stream)),
           "sdllm_sparse_attn_noalloc")


def sdllm_block_step(shape, step_in_block, delay, q_blk, k_in, v_in, idx, k_cache, v_cache, out, ws,
                     stream=None) -> int:
    st = ctypes.c_int32(-1)
    _check(load().sdllm_block_step(ctypes.byref(shape), step_in_block, delay, _ptr(q_blk), _ptr(k_in), _ptr(v_in),
                                   _ptr(idx), _ptr(k_cache), _ptr(v_cache), _ptr(out), _ptr(ws),
                                   ws.numel() * ws.element_size() if ws is not None else 0, _stream(stream),
                                   ctypes.byref(st)), "sdllm_block_step")
    return st.value


def sdllm_dense_attn(shape, q_full, k_full, v_full, out_full, stream=None) -> None:
    qs = (ctypes.c_int64 * 3)(*strides_of(q_full))
    os_ = (ctypes.c_int64 * 3)(*strides_of(out_full))
    _check(load().sdllm_dense_attn(ctypes.byref(shape), _ptr(q_full), qs, _ptr(k_full), _ptr(v_full), _ptr(out_full), os_,
                                   _stream(stream)), "sdllm_dense_attn")


def sdllm_stream_read_probe(src, sink=None, stream=None) -> None:
    _check(load().sdllm_stream_read_probe(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream(stream)),
           "sdllm_stream_read_probe")
