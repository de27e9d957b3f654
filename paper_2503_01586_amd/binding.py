"""Thin ctypes binding of libelitekv.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/elitekv.h).  Tensors are
torch tensors used purely as device memory; the stream is torch's current HIP stream unless one
is passed.  Nothing is computed here, and there is no fallback: if the library is missing the
import fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libelitekv.so")

ELITEKV_FP32 = 0
ELITEKV_BF16 = 1

OK, EINVAL, EINDEX, ENULL, EALIGN, EWORKSPACE, EUNSUPPORTED, EHIP, ESCRATCH = 0, -1, -2, -3, -4, -5, -6, -7, -8
NOALLOC_SCRATCH_BYTES = 32 << 20   # ELITEKV_NOALLOC_SCRATCH_BYTES


class elitekv_dims(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("r", C.c_int32), ("d_c", C.c_int32), ("dtype", C.c_int32), ("rope_base", C.c_double)]


class EliteKVError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, elitekv_strerror(status), status))


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "libelitekv.so is not built (%s). Run `python -c 'import __graft_entry__ as g; g.build()'` "
            "or `python paper_2503_01586_amd/build.py`." % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    P, I32, I64, SZ = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    DP = C.POINTER(elitekv_dims)
    sigs = {
        "elitekv_strerror": (C.c_char_p, [C.c_int]),
        "elitekv_cache_row_elems": (C.c_int, [DP, C.POINTER(I64), C.POINTER(I64)]),
        "elitekv_param_count": (C.c_int, [DP, C.POINTER(I64)]),
        "elitekv_validate_elite_idx": (C.c_int, [DP, P]),
        "elitekv_append_workspace_bytes": (SZ, [DP, I64]),
        "elitekv_append": (C.c_int, [DP, P, P, P, I64, P, P, P, P, P, I64, P, SZ, P]),
        "elitekv_decode_path": (C.c_int, [DP, I32]),
        "elitekv_decode_auto_splits": (I32, [DP, I64, I64]),
        "elitekv_decode_workspace_bytes": (SZ, [DP, I64, I64, I32]),
        "elitekv_decode_attn": (C.c_int, [DP, P, P, P, I64, I64, I64, P, P, P, P, P, I64, P, P, SZ, I32, P]),
        "elitekv_decode_attn_noalloc": (C.c_int, [DP, P, P, P, I64, I64, I64, P, P, P, P, P, I64, P, I32, P]),
        "elitekv_ropelite_search_workspace_bytes": (SZ, [I64, I32, I32, I32]),
        "elitekv_ropelite_search": (C.c_int, [P, P, P, I64, I32, I32, I32, C.c_double, P, P, P, SZ, P]),
        "elitekv_multiquery_workspace_bytes": (SZ, [DP, I64, I64, I64, I32]),
        "elitekv_multiquery_attn": (C.c_int, [DP, P, P, P, I64, I64, I64, I64, P, P, P, P, P, I64, P, P, SZ, I32, P]),
        "elitekv_prefill_attn_workspace_bytes": (SZ, [DP, I64, I64, I64]),
        "elitekv_prefill_attn": (C.c_int, [DP, P, P, P, I64, I64, I64, I64, P, P, P, P, P, I64, P, P, SZ, P]),
        "elitekv_slrd_param_count": (C.c_int, [DP, I32, C.POINTER(I64)]),
        "elitekv_slrd_append_workspace_bytes": (SZ, [DP, I32, I64]),
        "elitekv_slrd_append": (C.c_int, [DP, I32, P, P, P, I64, P, P, P, P, P, P, I64, P, SZ, P]),
        "elitekv_slrd_decode_workspace_bytes": (SZ, [DP, I32, I64, I64, I32]),
        "elitekv_slrd_decode_attn": (C.c_int, [DP, I32, P, P, P, I64, I64, I64, P, P, P, P, P, I64, P, P, SZ, I32,
                                               P]),
        "elitekv_slrd_multiquery_workspace_bytes": (SZ, [DP, I32, I64, I64, I64, I32]),
        "elitekv_slrd_multiquery_attn": (C.c_int, [DP, I32, P, P, P, I64, I64, I64, I64, P, P, P, P, P, I64, P, P, SZ,
                                                   I32, P]),
        "elitekv_slrd_prefill_attn_workspace_bytes": (SZ, [DP, I32, I64, I64, I64]),
        "elitekv_slrd_prefill_attn": (C.c_int, [DP, I32, P, P, P, I64, I64, I64, I64, P, P, P, P, P, I64, P, P, SZ, P]),
        "elitekv_decode_step_workspace_bytes": (SZ, [DP, I64, I64, I32]),
        "elitekv_decode_step": (C.c_int, [DP, P, P, P, P, P, I64, I64, I64, P, P, P, P, P, P, P, I64, P, P, SZ, I32,
                                          P]),
        "elitekv_block_step_workspace_bytes": (SZ, [DP, I64, I64, I32]),
        "elitekv_block_step": (C.c_int, [DP, P, P, P, P, I64, I64, I64, P, P, P, P, P, P, P, P, P, I64, P, P, SZ, I32, P]),
        "elitekv_slrd_block_step_workspace_bytes": (SZ, [DP, I32, I64, I64, I32]),
        "elitekv_slrd_block_step": (C.c_int, [DP, I32, P, P, P, P, I64, I64, I64, P, P, P, P, P, P, P, P, P, P, I64, P, P,
                                              SZ, I32, P]),
        "elitekv_slrd_decode_step_workspace_bytes": (SZ, [DP, I32, I64, I64, I32]),
        "elitekv_slrd_decode_step": (C.c_int, [DP, I32, P, P, P, P, P, I64, I64, I64, P, P, P, P, P, P, P, P, I64, P,
                                               P, SZ, I32, P]),
        "elitekv_decode_attn_stages": (C.c_int, [DP, P, P, P, I64, I64, I64, P, P, P, P, P, I64, P, P, SZ, I32,
                                                 P, I32, I32]),
        "elitekv_mha_decode_workspace_bytes": (SZ, [DP, I64, I64, I32]),
        "elitekv_mha_decode": (C.c_int, [DP, P, P, P, I64, I64, I64, P, P, I64, P, P, SZ, I32, P]),
        "elitekv_stream_read": (C.c_int, [P, SZ, P, P]),
        "elitekv_stream_read_mode": (C.c_int, [P, SZ, P, I32, C.POINTER(SZ), P]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib, tuple(sigs)


_lib, EXPORTS = _load()


def make_dims(d_model, n_heads, head_dim, r, d_c, dtype, rope_base=10000.0) -> elitekv_dims:
    if isinstance(dtype, str):
        dtype = {"fp32": ELITEKV_FP32, "bf16": ELITEKV_BF16}[dtype]
    elif isinstance(dtype, torch.dtype):
        dtype = {torch.float32: ELITEKV_FP32, torch.bfloat16: ELITEKV_BF16}[dtype]
    return elitekv_dims(int(d_model), int(n_heads), int(head_dim), int(r), int(d_c), int(dtype),
                        float(rope_base))


def torch_dtype(dims: elitekv_dims):
    return torch.float32 if dims.dtype == ELITEKV_FP32 else torch.bfloat16


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(status, where):
    if status != 0:
        raise EliteKVError(status, where)


def elitekv_strerror(status: int) -> str:
    return _lib.elitekv_strerror(int(status)).decode()


def elitekv_cache_row_elems(dims):
    ke, c = C.c_int64(), C.c_int64()
    _check(_lib.elitekv_cache_row_elems(C.byref(dims), C.byref(ke), C.byref(c)), "elitekv_cache_row_elems")
    return ke.value, c.value


def elitekv_param_count(dims) -> int:
    n = C.c_int64()
    _check(_lib.elitekv_param_count(C.byref(dims), C.byref(n)), "elitekv_param_count")
    return n.value


def elitekv_validate_elite_idx(dims, idx_host) -> int:
    """idx_host: a CPU int32 tensor / numpy array [n_h, r].  Returns the status (0 or EINDEX...)."""
    import numpy as np
    arr = np.ascontiguousarray(np.asarray(idx_host), dtype=np.int32)
    return _lib.elitekv_validate_elite_idx(C.byref(dims), arr.ctypes.data if arr.size else None)


def elitekv_append_workspace_bytes(dims, T) -> int:
    return _lib.elitekv_append_workspace_bytes(C.byref(dims), int(T))


def elitekv_append(dims, x, pos, slot, W_ke, W_dkv, elite_idx, ke_plane, c_plane, ws=None, stream=None,
                   T=None, plane_rows=None):
    T = x.shape[0] if T is None else T
    plane_rows = c_plane.shape[0] if plane_rows is None else plane_rows
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = _lib.elitekv_append(C.byref(dims), _ptr(x), _ptr(pos), _ptr(slot), int(T), _ptr(W_ke),
                             _ptr(W_dkv), _ptr(elite_idx), _ptr(ke_plane), _ptr(c_plane),
                             int(plane_rows), _ptr(ws), ws_bytes, _stream(stream))
    _check(st, "elitekv_append")


PATH_GENERIC, PATH_MATRIX_CORE = 0, 1


def elitekv_decode_path(dims, d_ck=0) -> int:
    """PATH_MATRIX_CORE or PATH_GENERIC (which kernels the decode entry points run for this shape)."""
    st = _lib.elitekv_decode_path(C.byref(dims), int(d_ck))
    if st < 0:
        raise EliteKVError(st, "elitekv_decode_path")
    return st


def elitekv_decode_auto_splits(dims, B, max_seq_len) -> int:
    return _lib.elitekv_decode_auto_splits(C.byref(dims), int(B), int(max_seq_len))


def elitekv_decode_workspace_bytes(dims, B, max_seq_len, n_splits=0) -> int:
    return _lib.elitekv_decode_workspace_bytes(C.byref(dims), int(B), int(max_seq_len), int(n_splits))


def elitekv_decode_attn(dims, q, q_pos, seq_len, max_seq_len, batch_stride_rows, W_uk, W_uv, elite_idx,
                        ke_plane, c_plane, out, ws, n_splits=0, stream=None, B=None, plane_rows=None):
    B = q.shape[0] if B is None else B
    plane_rows = c_plane.shape[0] if plane_rows is None else plane_rows
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = _lib.elitekv_decode_attn(C.byref(dims), _ptr(q), _ptr(q_pos), _ptr(seq_len), int(B),
                                  int(max_seq_len), int(batch_stride_rows), _ptr(W_uk), _ptr(W_uv),
                                  _ptr(elite_idx), _ptr(ke_plane), _ptr(c_plane), int(plane_rows),
                                  _ptr(out), _ptr(ws), ws_bytes, int(n_splits), _stream(stream))
    _check(st, "elitekv_decode_attn")


def elitekv_decode_attn_noalloc(dims, q, q_pos, seq_len, max_seq_len, batch_stride_rows, W_uk, W_uv, elite_idx,
                                ke_plane, c_plane, out, n_splits=0, stream=None, B=None, plane_rows=None):
    B = q.shape[0] if B is None else B
    plane_rows = c_plane.shape[0] if plane_rows is None else plane_rows
    st = _lib.elitekv_decode_attn_noalloc(C.byref(dims), _ptr(q), _ptr(q_pos), _ptr(seq_len), int(B),
                                          int(max_seq_len), int(batch_stride_rows), _ptr(W_uk), _ptr(W_uv),
                                          _ptr(elite_idx), _ptr(ke_plane), _ptr(c_plane), int(plane_rows),
                                          _ptr(out), int(n_splits), _stream(stream))
    _check(st, "elitekv_decode_attn_noalloc")


def elitekv_ropelite_search_workspace_bytes(T, n_heads, head_dim, r) -> int:
    return _lib.elitekv_ropelite_search_workspace_bytes(int(T), int(n_heads), int(head_dim), int(r))


def elitekv_ropelite_search(q, k, pos, r, rope_base, elite_out, dist_out, ws, stream=None):
    """q, k [T, n_h, d_h] float32; pos [T] int32; elite_out [n_h, r] int32; dist_out [n_h, r] float32 or None."""
    T, n_h, d_h = q.shape
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = _lib.elitekv_ropelite_search(_ptr(q), _ptr(k), _ptr(pos), int(T), int(n_h), int(d_h), int(r),
                                      float(rope_base), _ptr(elite_out), _ptr(dist_out), _ptr(ws), ws_bytes,
                                      _stream(stream))
    _check(st, "elitekv_ropelite_search")


def elitekv_multiquery_workspace_bytes(dims, B, T, max_seq_len, n_splits=0) -> int:
    return _lib.elitekv_multiquery_workspace_bytes(C.byref(dims), int(B), int(T), int(max_seq_len), int(n_splits))


def elitekv_multiquery_attn(dims, q, q_pos, kv_len, max_seq_len, batch_stride_rows, W_uk, W_uv, elite_idx, ke_plane,
                            c_plane, out, ws, n_splits=0, stream=None, plane_rows=None):
    """q [B, T, n_h, d_h]; q_pos, kv_len [B, T] (int32)."""
    B, T = q.shape[0], q.shape[1]
    plane_rows = c_plane.shape[0] if plane_rows is None else plane_rows
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = _lib.elitekv_multiquery_attn(C.byref(dims), _ptr(q), _ptr(q_pos), _ptr(kv_len), int(B), int(T),
                                      int(max_seq_len), int(batch_stride_rows), _ptr(W_uk), _ptr(W_uv),
                                      _ptr(elite_idx), _ptr(ke_plane), _ptr(c_plane), int(plane_rows), _ptr(out),
                                      _ptr(ws), ws_bytes, int(n_splits), _stream(stream))
    _check(st, "elitekv_multiquery_attn")


def elitekv_prefill_attn_workspace_bytes(dims, B, T, max_seq_len) -> int:
    return _lib.elitekv_prefill_attn_workspace_bytes(C.byref(dims), int(B), int(T), int(max_seq_len))


def elitekv_prefill_attn(dims, q, q_pos, kv_len, max_seq_len, batch_stride_rows, W_uk, W_uv, elite_idx, ke_plane,
                         c_plane, out, ws, stream=None, plane_rows=None):
    """q [B, T, n_h, d_h]; q_pos, kv_len [B, T] (int32)."""
    B, T = q.shape[0], q.shape[1]
    plane_rows = c_plane.shape[0] if plane_rows is None else plane_rows
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = _lib.elitekv_prefill_attn(C.byref(dims), _ptr(q), _ptr(q_pos), _ptr(kv_len), int(B), int(T),
                                   int(max_seq_len), int(batch_stride_rows), _ptr(W_uk), _ptr(W_uv),
                                   _ptr(elite_idx), _ptr(ke_plane), _ptr(c_plane), int(plane_rows), _ptr(out),
                                   _ptr(ws), ws_bytes, _stream(stream))
    _check(st, "elitekv_prefill_attn")


def elitekv_slrd_param_count(dims, d_ck) -> int:
    n = C.c_int64()
    _check(_lib.elitekv_slrd_param_count(C.byref(dims), int(d_ck), C.byref(n)), "elitekv_slrd_param_count")
    return n.value


def elitekv_slrd_append_workspace_bytes(dims, d_ck, T) -> int:
    return _lib.elitekv_slrd_append_workspace_bytes(C.byref(dims), int(d_ck), int(T))


def elitekv_slrd_append(dims, d_ck, x, pos, slot, W_ke, A_k, A_v, elite_idx, ke_plane, c_plane, ws=None,
                        stream=None, T=None, plane_rows=None):
    T = x.shape[0] if T is None else T
    plane_rows = c_plane.shape[0] if plane_rows is None else plane_rows
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = _lib.elitekv_slrd_append(C.byref(dims), int(d_ck), _ptr(x), _ptr(pos), _ptr(slot), int(T), _ptr(W_ke),
                                  _ptr(A_k), _ptr(A_v), _ptr(elite_idx), _ptr(ke_plane), _ptr(c_plane),
                                  int(plane_rows), _ptr(ws), ws_bytes, _stream(stream))
    _check(st, "elitekv_slrd_append")


def elitekv_slrd_decode_workspace_bytes(dims, d_ck, B, max_seq_len, n_splits=0) -> int:
    return _lib.elitekv_slrd_decode_workspace_bytes(C.byref(dims), int(d_ck), int(B), int(max_seq_len),
                                                    int(n_splits))


def elitekv_slrd_decode_attn(dims, d_ck, q, q_pos, seq_len, max_seq_len, batch_stride_rows, B_k, B_v, elite_idx,
                             ke_plane, c_plane, out, ws, n_splits=0, stream=None, B=None, plane_rows=None):
    B = q.shape[0] if B is None else B
    plane_rows = c_plane.shape[0] if plane_rows is None else plane_rows
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = _lib.elitekv_slrd_decode_attn(C.byref(dims), int(d_ck), _ptr(q), _ptr(q_pos), _ptr(seq_len), int(B),
                                       int(max_seq_len), int(batch_stride_rows), _ptr(B_k), _ptr(B_v),
                                       _ptr(elite_idx), _ptr(ke_plane), _ptr(c_plane), int(plane_rows),
                                       _ptr(out), _ptr(ws), ws_bytes, int(n_splits), _stream(stream))
    _check(st, "elitekv_slrd_decode_attn")


def elitekv_slrd_multiquery_workspace_bytes(dims, d_ck, B, T, max_seq_len, n_splits=0) -> int:
    return _lib.elitekv_slrd_multiquery_workspace_bytes(C.byref(dims), int(d_ck), int(B), int(T), int(max_seq_len),
                                                        int(n_splits))


def elitekv_slrd_multiquery_attn(dims, d_ck, q, q_pos, kv_len, max_seq_len, batch_stride_rows, B_k, B_v, elite_idx,
                                 ke_plane, c_plane, out, ws, n_splits=0, stream=None, plane_rows=None):
    """q [B, T, n_h, d_h]; q_pos, kv_len [B, T] (int32)."""
    B, T = q.shape[0], q.shape[1]
    plane_rows = c_plane.shape[0] if plane_rows is None else plane_rows
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = _lib.elitekv_slrd_multiquery_attn(C.byref(dims), int(d_ck), _ptr(q), _ptr(q_pos), _ptr(kv_len), int(B),
                                           int(T), int(max_seq_len), int(batch_stride_rows), _ptr(B_k), _ptr(B_v),
                                           _ptr(elite_idx), _ptr(ke_plane), _ptr(c_plane), int(plane_rows),
                                           _ptr(out), _ptr(ws), ws_bytes, int(n_splits), _stream(stream))
    _check(st, "elitekv_slrd_multiquery_attn")


def elitekv_slrd_prefill_attn_workspace_bytes(dims, d_ck, B, T, max_seq_len) -> int:
    return _lib.elitekv_slrd_prefill_attn_workspace_bytes(C.byref(dims), int(d_ck), int(B), int(T), int(max_seq_len))


def elitekv_slrd_prefill_attn(dims, d_ck, q, q_pos, kv_len, max_seq_len, batch_stride_rows, B_k, B_v, elite_idx,
                              ke_plane, c_plane, out, ws, stream=None, plane_rows=None):
    """q [B, T, n_h, d_h]; q_pos, kv_len [B, T] (int32)."""
    B, T = q.shape[0], q.shape[1]
    plane_rows = c_plane.shape[0] if plane_rows is None else plane_rows
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = _lib.elitekv_slrd_prefill_attn(C.byref(dims), int(d_ck), _ptr(q), _ptr(q_pos), _ptr(kv_len), int(B), int(T),
                                        int(max_seq_len), int(batch_stride_rows), _ptr(B_k), _ptr(B_v),
                                        _ptr(elite_idx), _ptr(ke_plane), _ptr(c_plane), int(plane_rows), _ptr(out),
                                        _ptr(ws), ws_bytes, _stream(stream))
    _check(st, "elitekv_slrd_prefill_attn")


def elitekv_decode_step_workspace_bytes(dims, B, max_seq_len, n_splits=0) -> int:
    return _lib.elitekv_decode_step_workspace_bytes(C.byref(dims), int(B), int(max_seq_len), int(n_splits))


def elitekv_decode_step(dims, x, q, pos, slot, seq_len, max_seq_len, batch_stride_rows, W_ke, W_dkv, W_uk, W_uv,
                        elite_idx, ke_plane, c_plane, out, ws, n_splits=0, stream=None, B=None, plane_rows=None):
    B = q.shape[0] if B is None else B
    plane_rows = c_plane.shape[0] if plane_rows is None else plane_rows
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = _lib.elitekv_decode_step(C.byref(dims), _ptr(x), _ptr(q), _ptr(pos), _ptr(slot), _ptr(seq_len), int(B),
                                  int(max_seq_len), int(batch_stride_rows), _ptr(W_ke), _ptr(W_dkv), _ptr(W_uk),
                                  _ptr(W_uv), _ptr(elite_idx), _ptr(ke_plane), _ptr(c_plane), int(plane_rows),
                                  _ptr(out), _ptr(ws), ws_bytes, int(n_splits), _stream(stream))
    _check(st, "elitekv_decode_step")


def elitekv_block_step_workspace_bytes(dims, B, max_seq_len, n_splits=0) -> int:
    return _lib.elitekv_block_step_workspace_bytes(C.byref(dims), int(B), int(max_seq_len), int(n_splits))


def elitekv_block_step(dims, x, pos, slot, seq_len, max_seq_len, batch_stride_rows, W_q, W_ke, W_dkv, W_uk, W_uv, W_o,
                       elite_idx, ke_plane, c_plane, y, ws, n_splits=0, stream=None, B=None, plane_rows=None):
    B = x.shape[0] if B is None else B
    plane_rows = c_plane.shape[0] if plane_rows is None else plane_rows
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = _lib.elitekv_block_step(C.byref(dims), _ptr(x), _ptr(pos), _ptr(slot), _ptr(seq_len), int(B),
                                 int(max_seq_len), int(batch_stride_rows), _ptr(W_q), _ptr(W_ke), _ptr(W_dkv),
                                 _ptr(W_uk), _ptr(W_uv), _ptr(W_o), _ptr(elite_idx), _ptr(ke_plane), _ptr(c_plane),
                                 int(plane_rows), _ptr(y), _ptr(ws), ws_bytes, int(n_splits), _stream(stream))
    _check(st, "elitekv_block_step")


def elitekv_slrd_block_step_workspace_bytes(dims, d_ck, B, max_seq_len, n_splits=0) -> int:
    return _lib.elitekv_slrd_block_step_workspace_bytes(C.byref(dims), int(d_ck), int(B), int(max_seq_len), int(n_splits))


def elitekv_slrd_block_step(dims, d_ck, x, pos, slot, seq_len, max_seq_len, batch_stride_rows, W_q, W_ke, A_k, A_v, B_k,
                            B_v, W_o, elite_idx, ke_plane, c_plane, y, ws, n_splits=0, stream=None, B=None,
                            plane_rows=None):
    B = x.shape[0] if B is None else B
    plane_rows = c_plane.shape[0] if plane_rows is None else plane_rows
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = _lib.elitekv_slrd_block_step(C.byref(dims), int(d_ck), _ptr(x), _ptr(pos), _ptr(slot), _ptr(seq_len), int(B),
                                      int(max_seq_len), int(batch_stride_rows), _ptr(W_q), _ptr(W_ke), _ptr(A_k),
                                      _ptr(A_v), _ptr(B_k), _ptr(B_v), _ptr(W_o), _ptr(elite_idx), _ptr(ke_plane),
                                      _ptr(c_plane), int(plane_rows), _ptr(y), _ptr(ws), ws_bytes, int(n_splits),
                                      _stream(stream))
    _check(st, "elitekv_slrd_block_step")


def elitekv_slrd_decode_step_workspace_bytes(dims, d_ck, B, max_seq_len, n_splits=0) -> int:
    return _lib.elitekv_slrd_decode_step_workspace_bytes(C.byref(dims), int(d_ck), int(B), int(max_seq_len),
                                                         int(n_splits))


def elitekv_slrd_decode_step(dims, d_ck, x, q, pos, slot, seq_len, max_seq_len, batch_stride_rows, W_ke, A_k, A_v,
                             B_k, B_v, elite_idx, ke_plane, c_plane, out, ws, n_splits=0, stream=None, B=None,
                             plane_rows=None):
    B = q.shape[0] if B is None else B
    plane_rows = c_plane.shape[0] if plane_rows is None else plane_rows
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = _lib.elitekv_slrd_decode_step(C.byref(dims), int(d_ck), _ptr(x), _ptr(q), _ptr(pos), _ptr(slot),
                                       _ptr(seq_len), int(B), int(max_seq_len), int(batch_stride_rows), _ptr(W_ke),
                                       _ptr(A_k), _ptr(A_v), _ptr(B_k), _ptr(B_v), _ptr(elite_idx), _ptr(ke_plane),
                                       _ptr(c_plane), int(plane_rows), _ptr(out), _ptr(ws), ws_bytes, int(n_splits),
                                       _stream(stream))
    _check(st, "elitekv_slrd_decode_step")


def elitekv_decode_attn_stages(dims, q, q_pos, seq_len, max_seq_len, batch_stride_rows, W_uk, W_uv, elite_idx,
                               ke_plane, c_plane, out, ws, stages, n_splits=0, stream=None, B=None,
                               plane_rows=None, d_ck=0):
    """stages: bit 0 query preparation, bit 1 split attention, bit 2 merge + up-projection.
    d_ck = 0: joint latent; d_ck > 0: separated latents (W_uk = B_k, W_uv = B_v)."""
    B = q.shape[0] if B is None else B
    plane_rows = c_plane.shape[0] if plane_rows is None else plane_rows
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = _lib.elitekv_decode_attn_stages(C.byref(dims), _ptr(q), _ptr(q_pos), _ptr(seq_len), int(B),
                                         int(max_seq_len), int(batch_stride_rows), _ptr(W_uk), _ptr(W_uv),
                                         _ptr(elite_idx), _ptr(ke_plane), _ptr(c_plane), int(plane_rows),
                                         _ptr(out), _ptr(ws), ws_bytes, int(n_splits), _stream(stream), int(stages),
                                         int(d_ck))
    _check(st, "elitekv_decode_attn_stages")


def elitekv_mha_decode_workspace_bytes(dims, B, max_seq_len, n_splits=0) -> int:
    return _lib.elitekv_mha_decode_workspace_bytes(C.byref(dims), int(B), int(max_seq_len), int(n_splits))


def elitekv_mha_decode(dims, q, q_pos, seq_len, max_seq_len, batch_stride_rows, k_plane, v_plane, out, ws,
                       n_splits=0, stream=None, B=None, plane_rows=None):
    B = q.shape[0] if B is None else B
    plane_rows = k_plane.shape[0] if plane_rows is None else plane_rows
    ws_bytes = 0 if ws is None else ws.numel() * ws.element_size()
    st = _lib.elitekv_mha_decode(C.byref(dims), _ptr(q), _ptr(q_pos), _ptr(seq_len), int(B),
                                 int(max_seq_len), int(batch_stride_rows), _ptr(k_plane), _ptr(v_plane),
                                 int(plane_rows), _ptr(out), _ptr(ws), ws_bytes, int(n_splits),
                                 _stream(stream))
    _check(st, "elitekv_mha_decode")


def elitekv_stream_read(src, sink, nbytes=None, stream=None):
    nbytes = src.numel() * src.element_size() if nbytes is None else nbytes
    st = _lib.elitekv_stream_read(_ptr(src), int(nbytes), _ptr(sink), _stream(stream))
    _check(st, "elitekv_stream_read")


def elitekv_stream_read_mode(src, sink, mode, nbytes=None, stream=None) -> int:
    """Returns the number of bytes the launch reads."""
    nbytes = src.numel() * src.element_size() if nbytes is None else nbytes
    n = C.c_size_t()
    st = _lib.elitekv_stream_read_mode(_ptr(src), int(nbytes), _ptr(sink), int(mode), C.byref(n), _stream(stream))
    _check(st, "elitekv_stream_read_mode")
    return int(n.value)


def raw():
    """The ctypes library handle, for tests that exercise the error paths with raw pointers."""
    return _lib
