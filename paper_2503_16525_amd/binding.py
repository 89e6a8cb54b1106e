"""ctypes binding of libkvshare_hip.so: argument marshalling only.

Every function here has the name and the semantics of the C entry point declared in
``include/kvs.h``; tensors are torch CUDA tensors (device memory and streams are all torch is
used for), host-side tables are python sequences.  There is no CPU fallback: if the library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libkvshare_hip.so")

F32, BF16 = 0, 1
SCORE_V, SCORE_KV = 0, 1
OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP = 0, 1, 2, 3, 4

EXPORTS = ("kvs_deviation", "kvs_deviation_topk", "kvs_select_topk", "kvs_select_topk_static", "kvs_scatter_kv", "kvs_partial_attention",
           "kvs_decode_check", "kvs_attn_colsum", "kvs_first_order_impact", "kvs_match_tokens", "kvs_project_qkv", "kvs_workspace_size", "kvs_strerror", "kvs_last_error", "kvs_version")


class KvsError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str):
        super().__init__(f"{where}: status {status}: {detail}")
        self.status = status


class Shape(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32)]


_lib: Optional[ctypes.CDLL] = None


def load(build_if_missing: bool = True) -> ctypes.CDLL:
    """Loads the in-tree library; builds it first only when no built library exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise FileNotFoundError(LIB_PATH)
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    sp = ctypes.POINTER(Shape)
    lib.kvs_deviation.argtypes = [sp, i64, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp]
    lib.kvs_deviation_topk.argtypes = [sp, i64, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, i32, vp, vp, sz, vp]
    lib.kvs_select_topk.argtypes = [vp, i32, vp, vp, vp, vp, sz, vp]
    lib.kvs_select_topk_static.argtypes = [vp, i32, vp, vp, vp, vp]
    lib.kvs_scatter_kv.argtypes = [sp, i64, vp, vp, vp, i64, vp, vp, vp, vp, vp]
    lib.kvs_partial_attention.argtypes = [sp, i32, vp, vp, vp, vp, vp, vp, vp, f32, vp, vp, vp, sz, vp]
    lib.kvs_decode_check.argtypes = [sp, i32, i64, vp, vp, vp, vp, vp, vp, vp, f32, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_attn_colsum.argtypes = [sp, i64, vp, vp, f32, vp, vp, sz, vp]
    lib.kvs_first_order_impact.argtypes = [sp, i64, vp, vp, vp, vp, vp, vp, vp, vp, f32, vp, vp, vp, vp, sz, vp]
    lib.kvs_match_tokens.argtypes = [vp, i64, vp, i64, i32, ctypes.c_uint32, ctypes.c_uint32, vp, vp, vp, vp, vp, sz, vp]
    lib.kvs_project_qkv.argtypes = [sp, i32, vp, i64, vp, vp, i64, vp, vp, i64, vp, vp, vp, vp]
    lib.kvs_workspace_size.argtypes = [ctypes.c_char_p, sp, i32, i64, i64]
    for n in ("kvs_deviation", "kvs_deviation_topk", "kvs_select_topk", "kvs_select_topk_static", "kvs_scatter_kv", "kvs_partial_attention",
              "kvs_decode_check", "kvs_attn_colsum", "kvs_first_order_impact", "kvs_match_tokens", "kvs_project_qkv"):
        getattr(lib, n).restype = ctypes.c_int
    lib.kvs_workspace_size.restype = sz
    lib.kvs_strerror.argtypes = [ctypes.c_int]
    for n in ("kvs_strerror", "kvs_last_error", "kvs_version"):
        getattr(lib, n).restype = ctypes.c_char_p
    _lib = lib
    return lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _ptr(t: Optional[torch.Tensor], dtype: Optional[torch.dtype] = None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise TypeError("device tensor expected")
    if not t.is_contiguous():
        raise TypeError("contiguous tensor expected")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _host(seq, dtype) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(seq, dtype=dtype))


def _hp(a: np.ndarray) -> int:
    return a.ctypes.data


def _check(rc: int, where: str) -> None:
    if rc != OK:
        raise KvsError(rc, where, load().kvs_last_error().decode())


def last_error() -> str:
    return load().kvs_last_error().decode()


def make_shape(n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: int) -> Shape:
    return Shape(n_q_heads, n_kv_heads, head_dim, dtype)


def kvs_workspace_size(call: str, shape: Optional[Shape], batch: int, n_rows_total: int, n_sel_total: int = 0) -> int:
    return int(load().kvs_workspace_size(call.encode(), ctypes.byref(shape) if shape is not None else None, batch,
                                         n_rows_total, n_sel_total))


def kvs_deviation(shape: Shape, n_tokens: int, k_fresh, v_fresh, k_cache, v_cache, reused, alpha,
                  mode: int, dev_k, dev_v, score, stream=None) -> None:
    rc = load().kvs_deviation(ctypes.byref(shape), n_tokens, _ptr(k_fresh), _ptr(v_fresh), _ptr(k_cache),
                              _ptr(v_cache), _ptr(reused, torch.uint8), _ptr(alpha, torch.float32), mode,
                              _ptr(dev_k, torch.float32), _ptr(dev_v, torch.float32),
                              _ptr(score, torch.float32), _stream(stream))
    _check(rc, "kvs_deviation")


def kvs_deviation_topk(shape: Shape, n_tokens: int, k_fresh, v_fresh, k_cache, v_cache, reused, alpha,
                       mode: int, dev_k, dev_v, score, k: int, idx_out, workspace=None, stream=None) -> None:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = load().kvs_deviation_topk(ctypes.byref(shape), n_tokens, _ptr(k_fresh), _ptr(v_fresh), _ptr(k_cache),
                                   _ptr(v_cache), _ptr(reused, torch.uint8), _ptr(alpha, torch.float32), mode,
                                   _ptr(dev_k, torch.float32), _ptr(dev_v, torch.float32),
                                   _ptr(score, torch.float32), k, _ptr(idx_out, torch.int32), _ptr(workspace),
                                   ws_bytes, _stream(stream))
    _check(rc, "kvs_deviation_topk")


def kvs_select_topk(scores, row_off: Sequence[int], k_row: Sequence[int], idx_out,
                    workspace=None, stream=None) -> None:
    ro, kr = _host(row_off, np.int64), _host(k_row, np.int32)
    if len(ro) != len(kr) + 1:
        raise ValueError("row_off must have len(k_row)+1 entries")
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = load().kvs_select_topk(_ptr(scores, torch.float32), len(kr), _hp(ro), _hp(kr),
                                _ptr(idx_out, torch.int32), _ptr(workspace), ws_bytes, _stream(stream))
    _check(rc, "kvs_select_topk")


def kvs_select_topk_static(scores, row_off: Sequence[int], k_row: Sequence[int], idx_out, stream=None) -> None:
    ro, kr = _host(row_off, np.int64), _host(k_row, np.int32)
    if len(ro) != len(kr) + 1:
        raise ValueError("row_off must have len(k_row)+1 entries")
    rc = load().kvs_select_topk_static(_ptr(scores, torch.float32), len(kr), _hp(ro), _hp(kr),
                                       _ptr(idx_out, torch.int32), _stream(stream))
    _check(rc, "kvs_select_topk_static")


def kvs_scatter_kv(shape: Shape, n_rows: int, k_new, v_new, sel_pos, n_sel: int, k_cache, v_cache,
                   reused=None, dev_v=None, stream=None) -> None:
    rc = load().kvs_scatter_kv(ctypes.byref(shape), n_rows, _ptr(k_new), _ptr(v_new),
                               _ptr(sel_pos, torch.int32), n_sel, _ptr(k_cache), _ptr(v_cache),
                               _ptr(reused, torch.uint8), _ptr(dev_v, torch.float32), _stream(stream))
    _check(rc, "kvs_scatter_kv")


def kvs_partial_attention(shape: Shape, ctx_off: Sequence[int], ctx_len: Sequence[int], cu_sel: Sequence[int],
                          q_sel, sel_pos, k_cache, v_cache, scale: float, out, lse_out=None,
                          workspace=None, stream=None) -> None:
    co, cl, cs = _host(ctx_off, np.int64), _host(ctx_len, np.int64), _host(cu_sel, np.int64)
    if len(co) != len(cl) or len(cs) != len(co) + 1:
        raise ValueError("ctx_off/ctx_len need one entry per request and cu_sel one more")
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = load().kvs_partial_attention(ctypes.byref(shape), len(co), _hp(co), _hp(cl), _hp(cs), _ptr(q_sel),
                                      _ptr(sel_pos, torch.int32), _ptr(k_cache), _ptr(v_cache), scale,
                                      _ptr(out), _ptr(lse_out, torch.float32), _ptr(workspace), ws_bytes,
                                      _stream(stream))
    _check(rc, "kvs_partial_attention")


def kvs_decode_check(shape: Shape, n_rows: int, ctx_off: Sequence[int], ctx_len: Sequence[int], q_new,
                     k_cache, v_cache, dev_v, reused, scale: float, k_req: Sequence[int], idx_out,
                     score_out=None, attn_out=None, workspace=None, stream=None) -> None:
    co, cl, kr = _host(ctx_off, np.int64), _host(ctx_len, np.int64), _host(k_req, np.int32)
    if not (len(co) == len(cl) == len(kr)):
        raise ValueError("ctx_off, ctx_len and k_req need one entry per request")
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = load().kvs_decode_check(ctypes.byref(shape), len(co), n_rows, _hp(co), _hp(cl), _ptr(q_new),
                                 _ptr(k_cache), _ptr(v_cache), _ptr(dev_v, torch.float32),
                                 _ptr(reused, torch.uint8), scale, _hp(kr), _ptr(idx_out, torch.int32),
                                 _ptr(score_out, torch.float32), _ptr(attn_out), _ptr(workspace), ws_bytes,
                                 _stream(stream))
    _check(rc, "kvs_decode_check")


def kvs_attn_colsum(shape: Shape, n_tokens: int, q, k, scale: float, alpha, workspace, stream=None) -> None:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = load().kvs_attn_colsum(ctypes.byref(shape), n_tokens, _ptr(q), _ptr(k), scale, _ptr(alpha, torch.float32),
                                _ptr(workspace), ws_bytes, _stream(stream))
    _check(rc, "kvs_attn_colsum")


def kvs_first_order_impact(shape: Shape, n_tokens: int, q, k_fresh, v_fresh, k_cache, v_cache, h_fresh, lse, reused,
                           scale: float, impact_v, impact_k, impact_kv, workspace, stream=None) -> None:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = load().kvs_first_order_impact(ctypes.byref(shape), n_tokens, _ptr(q), _ptr(k_fresh), _ptr(v_fresh), _ptr(k_cache),
                                       _ptr(v_cache), _ptr(h_fresh), _ptr(lse, torch.float32), _ptr(reused, torch.uint8),
                                       scale, _ptr(impact_v, torch.float32), _ptr(impact_k, torch.float32),
                                       _ptr(impact_kv, torch.float32), _ptr(workspace), ws_bytes, _stream(stream))
    _check(rc, "kvs_first_order_impact")


def kvs_match_tokens(target, candidate, window: int, hash_base: int, hash_modulus: int, match_cand,
                     target_matches, candidate_matches, n_matches, workspace, stream=None) -> None:
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = load().kvs_match_tokens(_ptr(target, torch.int32), target.numel() if target is not None else 0,
                                 _ptr(candidate, torch.int32), candidate.numel() if candidate is not None else 0,
                                 window, hash_base, hash_modulus, _ptr(match_cand, torch.int32),
                                 _ptr(target_matches, torch.int32), _ptr(candidate_matches, torch.int32),
                                 _ptr(n_matches, torch.int64), _ptr(workspace), ws_bytes, _stream(stream))
    _check(rc, "kvs_match_tokens")


def kvs_project_qkv(shape: Shape, x, x_rows, sel_pos, n_sel: int, w_qkv, rope, q_out, k_out, v_out, stream=None) -> None:
    rc = load().kvs_project_qkv(ctypes.byref(shape), x.shape[1], _ptr(x), x.shape[0], _ptr(x_rows, torch.int32),
                                _ptr(sel_pos, torch.int32), n_sel, _ptr(w_qkv), _ptr(rope, torch.float32),
                                rope.shape[0] if rope is not None else 0, _ptr(q_out), _ptr(k_out), _ptr(v_out), _stream(stream))
    _check(rc, "kvs_project_qkv")


def shape_of(workload) -> Shape:
    """kvs_shape of a synth.Workload."""
    return Shape(workload.n_q_heads, workload.n_kv_heads, workload.head_dim,
                 F32 if workload.dtype == "f32" else BF16)
