"""ctypes binding for libdapq.so.  Function names and argument order follow include/dapq.h.

torch is used for device memory and streams only: tensors are passed down as raw pointers, the
current torch stream as the hipStream_t.  Nothing here computes anything.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
# DAPQ_LIBRARY names another build of the same library (the host-sanitized one the tests make); there is no other
# implementation to fall back to
_LIB_PATH = os.environ.get("DAPQ_LIBRARY") or os.path.join(_PKG, "libdapq.so")
_lib = None

EXPORTS = (
    "dapq_workspace_bytes", "dapq_last_error", "dapq_rope_apply", "dapq_pseudo_tokens", "dapq_pseudo_queries", "dapq_pseudo_queries_workspace_bytes", "dapq_score", "dapq_score_stats",
    "dapq_score_accumulate", "dapq_score_stats_extend", "dapq_pool", "dapq_topk", "dapq_pool_topk", "dapq_topk_workspace_bytes", "dapq_gather", "dapq_recall", "dapq_decode_attention",
    "dapq_score_static", "dapq_score_static_capacity", "dapq_score_single_launch",
)


class DapqError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libdapq error {code}: {message}")
        self.code = code


class Shape(C.Structure):
    """Mirror of `dapq_shape`."""
    _fields_ = [
        ("n_layers", C.c_int32), ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("n_pseudo", C.c_int32), ("total_tokens", C.c_int64),
        ("cu_seqlens", C.c_void_p),
        ("k_stride_layer", C.c_int64), ("k_stride_seq", C.c_int64), ("k_stride_head", C.c_int64),
        ("k_stride_token", C.c_int64),
        ("v_stride_layer", C.c_int64), ("v_stride_seq", C.c_int64), ("v_stride_head", C.c_int64),
        ("v_stride_token", C.c_int64),
        ("q_stride_layer", C.c_int64), ("q_stride_seq", C.c_int64), ("q_stride_head", C.c_int64),
        ("q_stride_row", C.c_int64),
        ("scale", C.c_float),
    ]


class Qproj(C.Structure):
    """Mirror of `dapq_qproj`."""
    _fields_ = [
        ("n_layers", C.c_int32), ("rows", C.c_int32), ("hidden", C.c_int32), ("n_q_heads", C.c_int32),
        ("head_dim", C.c_int32), ("total_tokens", C.c_int64),
        ("x_stride_layer", C.c_int64), ("x_stride_token", C.c_int64),
        ("w_stride_layer", C.c_int64), ("w_stride_row", C.c_int64),
        ("q_stride_layer", C.c_int64), ("q_stride_head", C.c_int64), ("q_stride_row", C.c_int64),
    ]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libdapq.so (built in-tree by paper_2603_11564_amd/build.py).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is not built; run `python -m paper_2603_11564_amd.build` "
                          "(there is no fallback path)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    sp = C.POINTER(Shape)
    lib.dapq_workspace_bytes.restype = sz
    lib.dapq_workspace_bytes.argtypes = [sp]
    lib.dapq_last_error.restype = C.c_char_p
    lib.dapq_last_error.argtypes = []
    lib.dapq_rope_apply.argtypes = [vp, vp, vp, i64, i32, i32, i64, i64, C.c_double, i32, vp]
    lib.dapq_pseudo_tokens.argtypes = [sp, i32, i32, vp, vp, vp]
    lib.dapq_pseudo_queries.argtypes = [C.POINTER(Qproj), vp, vp, vp, vp, C.c_double, i32, vp, vp, sz, vp]
    lib.dapq_pseudo_queries_workspace_bytes.argtypes = [C.POINTER(Qproj)]
    lib.dapq_score.argtypes = [sp, vp, vp, vp, vp, sz, vp]
    lib.dapq_score_stats.argtypes = [sp, vp, vp, vp, vp, sz, vp]
    lib.dapq_score_accumulate.argtypes = [sp, vp, vp, vp, vp, vp, sz, vp]
    lib.dapq_score_stats_extend.argtypes = [sp, vp, vp, i64, i64, i64, i64, vp, vp]
    lib.dapq_pool.argtypes = [sp, vp, vp, i32, vp]
    lib.dapq_topk.argtypes = [sp, vp, i32, vp, vp, vp, vp, sz, vp]
    lib.dapq_pool_topk.argtypes = [sp, vp, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.dapq_topk_workspace_bytes.argtypes = [sp, i32]
    lib.dapq_gather.argtypes = [sp, vp, vp, vp, vp, i32, vp, vp, vp]
    lib.dapq_recall.argtypes = [sp, vp, vp, i32, vp, vp, i32, vp, vp, vp]
    lib.dapq_decode_attention.argtypes = [sp, vp, vp, vp, vp, i32, vp, vp]
    lib.dapq_score_static.argtypes = [sp, vp, vp, vp, vp]
    lib.dapq_score_static_capacity.argtypes = []
    lib.dapq_score_single_launch.argtypes = [sp]
    for name in EXPORTS[2:]:
        getattr(lib, name).restype = C.c_int
    lib.dapq_pseudo_queries_workspace_bytes.restype = sz
    lib.dapq_score_static_capacity.restype = sz
    lib.dapq_topk_workspace_bytes.restype = sz
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise DapqError(rc, load_library().dapq_last_error().decode())


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is not None:
        return stream if isinstance(stream, int) else stream.cuda_stream
    import torch
    return torch.cuda.current_stream().cuda_stream


def make_shape(*, n_layers, batch, n_q_heads, n_kv_heads, n_pseudo, total_tokens, head_dim=128, cu_seqlens=None,
               k_strides=(0, 0, 0, 0), v_strides=(0, 0, 0, 0), q_strides=(0, 0, 0, 0), scale) -> Shape:
    """Strides are (layer, seq, head, token|row) in elements.  cu_seqlens: device int32 tensor or None.
    scale: the softmax scale 1/sqrt(d_k) of App. C.1, as a number: the caller supplies it, nothing is computed here."""
    s = Shape()
    s.n_layers, s.batch, s.n_q_heads, s.n_kv_heads = n_layers, batch, n_q_heads, n_kv_heads
    s.head_dim, s.n_pseudo, s.total_tokens = head_dim, n_pseudo, total_tokens
    s.cu_seqlens = _ptr(cu_seqlens)
    s.k_stride_layer, s.k_stride_seq, s.k_stride_head, s.k_stride_token = k_strides
    s.v_stride_layer, s.v_stride_seq, s.v_stride_head, s.v_stride_token = v_strides
    s.q_stride_layer, s.q_stride_seq, s.q_stride_head, s.q_stride_row = q_strides
    s.scale = float(scale)
    s._keepalive = cu_seqlens
    return s


def workspace_bytes(shape: Shape) -> int:
    return int(load_library().dapq_workspace_bytes(C.byref(shape)))


def dapq_rope_apply(x_in, x_out, pos, rows, heads, head_dim, stride_row, stride_head, theta, pairing=0,
                    stream=None):
    _check(load_library().dapq_rope_apply(_ptr(x_in), _ptr(x_out), _ptr(pos), rows, heads, head_dim, stride_row,
                                          stride_head, float(theta), pairing, _stream(stream)))


def dapq_score(shape, q, k, scores, workspace, stream=None):
    _check(load_library().dapq_score(C.byref(shape), _ptr(q), _ptr(k), _ptr(scores), _ptr(workspace),
                                     0 if workspace is None else workspace.numel() * workspace.element_size(),
                                     _stream(stream)))


def score_single_launch(shape) -> bool:
    """Whether dapq_score runs both passes of this shape in one kernel."""
    rc = load_library().dapq_score_single_launch(C.byref(shape))
    if rc < 0:
        _check(rc)
    return bool(rc)


def dapq_score_static(shape, q, k, scores, stream=None):
    _check(load_library().dapq_score_static(C.byref(shape), _ptr(q), _ptr(k), _ptr(scores), _stream(stream)))


def score_static_capacity() -> int:
    return int(load_library().dapq_score_static_capacity())


def dapq_score_stats(shape, q, k, lse2, workspace, stream=None):
    _check(load_library().dapq_score_stats(C.byref(shape), _ptr(q), _ptr(k), _ptr(lse2), _ptr(workspace),
                                           0 if workspace is None else workspace.numel() * workspace.element_size(),
                                           _stream(stream)))


def dapq_score_accumulate(shape, q, k, lse2, scores, workspace, stream=None):
    _check(load_library().dapq_score_accumulate(
        C.byref(shape), _ptr(q), _ptr(k), _ptr(lse2), _ptr(scores), _ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream)))


def dapq_score_stats_extend(shape, q, k_pseudo, kp_strides, lse2, stream=None):
    """kp_strides = (layer, seq, head, row) in elements."""
    sl, ss, sh, sr = kp_strides
    _check(load_library().dapq_score_stats_extend(C.byref(shape), _ptr(q), _ptr(k_pseudo), sl, ss, sh, sr, _ptr(lse2),
                                                  _stream(stream)))


def dapq_pool(shape, scores, pooled, width=7, stream=None):
    _check(load_library().dapq_pool(C.byref(shape), _ptr(scores), _ptr(pooled), width, _stream(stream)))


def dapq_topk(shape, pooled, budget, budget_per_seq, idx, count, workspace=None, stream=None):
    _check(load_library().dapq_topk(C.byref(shape), _ptr(pooled), budget, _ptr(budget_per_seq), _ptr(idx),
                                    _ptr(count), _ptr(workspace),
                                    0 if workspace is None else workspace.numel() * workspace.element_size(),
                                    _stream(stream)))


def dapq_pool_topk(shape, scores, width, budget, budget_per_seq, idx, count, pooled=None, stream=None, workspace=None):
    _check(load_library().dapq_pool_topk(C.byref(shape), _ptr(scores), width, budget, _ptr(budget_per_seq), _ptr(idx),
                                         _ptr(count), _ptr(pooled), _ptr(workspace),
                                         0 if workspace is None else workspace.numel() * workspace.element_size(),
                                         _stream(stream)))


def topk_workspace_bytes(shape, budget) -> int:
    """Bytes of the optional workspace of dapq_topk / dapq_pool_topk (0: no head is long enough to need it)."""
    return int(load_library().dapq_topk_workspace_bytes(C.byref(shape), budget))


def dapq_gather(shape, k, v, idx, count, budget, k_out, v_out, stream=None):
    _check(load_library().dapq_gather(C.byref(shape), _ptr(k), _ptr(v), _ptr(idx), _ptr(count), budget,
                                      _ptr(k_out), _ptr(v_out), _stream(stream)))


def dapq_recall(shape, idx_gold, count_gold, budget_gold, idx_pred, count_pred, budget_pred, common, recall=None,
                stream=None):
    _check(load_library().dapq_recall(C.byref(shape), _ptr(idx_gold), _ptr(count_gold), budget_gold, _ptr(idx_pred),
                                      _ptr(count_pred), budget_pred, _ptr(common), _ptr(recall), _stream(stream)))


def dapq_decode_attention(shape, q_decode, k_cache, v_cache, count, budget, out, stream=None):
    _check(load_library().dapq_decode_attention(C.byref(shape), _ptr(q_decode), _ptr(k_cache), _ptr(v_cache), _ptr(count),
                                                budget, _ptr(out), _stream(stream)))


def dapq_pseudo_tokens(shape, first_m, last_n, token_idx, positions, stream=None):
    _check(load_library().dapq_pseudo_tokens(C.byref(shape), first_m, last_n, _ptr(token_idx), _ptr(positions),
                                             _stream(stream)))


def pseudo_queries_workspace_bytes(desc) -> int:
    return int(load_library().dapq_pseudo_queries_workspace_bytes(C.byref(desc)))


def dapq_pseudo_queries(desc, x, token_idx, w_q, positions, theta, pairing, q_out, workspace=None, stream=None):
    _check(load_library().dapq_pseudo_queries(C.byref(desc), _ptr(x), _ptr(token_idx), _ptr(w_q), _ptr(positions),
                                              float(theta), int(pairing), _ptr(q_out), _ptr(workspace),
                                              0 if workspace is None else workspace.numel() * workspace.element_size(),
                                              _stream(stream)))
