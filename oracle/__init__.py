"""CPU oracle for the DHD KV-reuse hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes marshalling around ``oracle/kvso.c`` (plain C, double accumulators, OpenMP over
independent tokens/queries).  Only tests, the smoke check and the benchmark's cpu_baseline leg
may import this package; the GPU library never does, and this package never imports the GPU
library.  All arithmetic lives in the C file; nothing here computes anything.

Tensors are numpy arrays or CPU torch tensors.  bf16 data travels as its raw 16-bit pattern.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

try:  # torch is optional here: numpy inputs work without it
    import torch
except Exception:  # pragma: no cover
    torch = None

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvso.c")
_LIB = os.path.join(_HERE, "libkvso.so")

F32, BF16 = 0, 1
SCORE_V, SCORE_KV = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE: no fast-math, so sums keep their order)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Shape(ctypes.Structure):
    _fields_ = [("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32)]


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        for name in ("kvso_deviation", "kvso_alpha_prefill", "kvso_select_topk", "kvso_scatter_kv",
                     "kvso_partial_attention", "kvso_decode_check", "kvso_first_order_impact", "kvso_exact_impact",
                     "kvso_window_hash", "kvso_match_tokens", "kvso_schedule", "kvso_project_qkv", "kvso_max_threads"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def max_threads() -> int:
    return int(lib().kvso_max_threads())


# ---- marshalling helpers -------------------------------------------------------------------

def _as_np(x, want: Optional[np.dtype] = None) -> Optional[np.ndarray]:
    """numpy view of a tensor; bf16 torch tensors become uint16 bit patterns."""
    if x is None:
        return None
    if torch is not None and isinstance(x, torch.Tensor):
        x = x.detach().cpu().contiguous()
        if x.dtype == torch.bfloat16:
            x = x.view(torch.int16).numpy().view(np.uint16)
        else:
            x = x.numpy()
    a = np.ascontiguousarray(x)
    if want is not None and a.dtype != want:
        a = np.ascontiguousarray(a.astype(want))
    return a


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"K/V/Q must be float32 or bf16 bit patterns, got {a.dtype}")


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _shape(n_q_heads: int, n_kv_heads: int, head_dim: int, code: int) -> _Shape:
    return _Shape(n_q_heads, n_kv_heads, head_dim, code)


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle {what}: invalid argument")


# ---- the calls -----------------------------------------------------------------------------

def deviation(v_fresh, v_cache, k_fresh=None, k_cache=None, reused=None, alpha=None,
              mode: int = SCORE_V, n_q_heads: Optional[int] = None, want_dev_k: bool = False):
    """-> (dev_k or None, dev_v, score); dev_* float32 [Hkv, N], score float32 [N]."""
    vf, vc = _as_np(v_fresh), _as_np(v_cache)
    kf, kc = _as_np(k_fresh), _as_np(k_cache)
    n, hk, d = vf.shape
    code = _dtype_code(vf)
    sh = _shape(n_q_heads or hk, hk, d, code)
    ru = _as_np(reused, np.uint8)
    al = _as_np(alpha, np.float32)
    dev_v = np.empty((hk, n), np.float32)
    dev_k = np.empty((hk, n), np.float32) if (want_dev_k or mode == SCORE_KV) else None
    score = np.empty((n,), np.float32)
    rc = lib().kvso_deviation(ctypes.byref(sh), ctypes.c_int64(n), _p(kf), _p(vf), _p(kc), _p(vc),
                              _p(ru), _p(al), ctypes.c_int(mode), _p(dev_k), _p(dev_v), _p(score))
    _check(rc, "deviation")
    return dev_k, dev_v, score


def alpha_prefill(q, k, scale: float):
    """-> (alpha_h float64 [Hq, N], alpha_g float64 [Hkv, N])."""
    qa, ka = _as_np(q), _as_np(k)
    n, hq, d = qa.shape
    hk = ka.shape[1]
    sh = _shape(hq, hk, d, _dtype_code(qa))
    ah = np.empty((hq, n), np.float64)
    ag = np.empty((hk, n), np.float64)
    rc = lib().kvso_alpha_prefill(ctypes.byref(sh), ctypes.c_int64(n), _p(qa), _p(ka),
                                  ctypes.c_double(scale), _p(ah), _p(ag))
    _check(rc, "alpha_prefill")
    return ah, ag


def select_topk(scores, row_off: Sequence[int], k_row: Sequence[int]) -> np.ndarray:
    """-> int32 indices, row-local, ascending within each row, rows packed back to back."""
    sc = _as_np(scores, np.float32)
    ro = np.ascontiguousarray(np.asarray(row_off, dtype=np.int64))
    kr = np.ascontiguousarray(np.asarray(k_row, dtype=np.int32))
    out = np.empty((int(kr.sum()),), np.int32)
    rc = lib().kvso_select_topk(_p(sc), ctypes.c_int32(len(kr)), _p(ro), _p(kr), _p(out))
    _check(rc, "select_topk")
    return out


def scatter_kv(k_new, v_new, sel_pos, k_cache: np.ndarray, v_cache: np.ndarray,
               reused: Optional[np.ndarray] = None, dev_v: Optional[np.ndarray] = None) -> None:
    """In place on the numpy arrays k_cache, v_cache, reused, dev_v."""
    for a in (k_cache, v_cache, reused, dev_v):
        if a is not None and not (isinstance(a, np.ndarray) and a.flags.c_contiguous and a.flags.writeable):
            raise TypeError("scatter_kv updates contiguous writable numpy arrays in place")
    kn, vn = _as_np(k_new), _as_np(v_new)
    sp = _as_np(sel_pos, np.int32)
    rows, hk, d = k_cache.shape
    sh = _shape(hk, hk, d, _dtype_code(k_cache))
    if kn.dtype != k_cache.dtype:
        raise TypeError("k_new dtype differs from the cache")
    rc = lib().kvso_scatter_kv(ctypes.byref(sh), ctypes.c_int64(rows), _p(kn), _p(vn), _p(sp),
                               ctypes.c_int64(len(sp)), _p(k_cache), _p(v_cache), _p(reused), _p(dev_v))
    _check(rc, "scatter_kv")


def partial_attention(q_sel, sel_pos, k_cache, v_cache, scale: float,
                      ctx_off: Optional[Sequence[int]] = None, ctx_len: Optional[Sequence[int]] = None,
                      cu_sel: Optional[Sequence[int]] = None):
    """-> (out float64 [n_sel, Hq, d], lse float64 [n_sel, Hq]).  Single request by default."""
    qa, ka, va = _as_np(q_sel), _as_np(k_cache), _as_np(v_cache)
    sp = _as_np(sel_pos, np.int32)
    ns, hq, d = qa.shape
    rows, hk, _ = ka.shape
    if ctx_off is None:
        ctx_off, ctx_len, cu_sel = [0], [rows], [0, ns]
    co = np.ascontiguousarray(np.asarray(ctx_off, dtype=np.int64))
    cl = np.ascontiguousarray(np.asarray(ctx_len, dtype=np.int64))
    cs = np.ascontiguousarray(np.asarray(cu_sel, dtype=np.int64))
    sh = _shape(hq, hk, d, _dtype_code(qa))
    out = np.empty((ns, hq, d), np.float64)
    lse = np.empty((ns, hq), np.float64)
    rc = lib().kvso_partial_attention(ctypes.byref(sh), ctypes.c_int32(len(co)), _p(co), _p(cl), _p(cs),
                                      _p(qa), _p(sp), _p(ka), _p(va), ctypes.c_double(scale),
                                      _p(out), _p(lse))
    _check(rc, "partial_attention")
    return out, lse


def first_order_impact(q, k_fresh, v_fresh, k_cache, v_cache, scale: float, reused=None):
    """-> (impact_v, impact_k, impact_kv), float32 [N] each: the first-order movement of the attention
    output that reusing token i causes, value direction, key direction and both (small N only)."""
    qa = _as_np(q)
    kf, vf, kc, vc = _as_np(k_fresh), _as_np(v_fresh), _as_np(k_cache), _as_np(v_cache)
    n, hq, d = qa.shape
    hk = kf.shape[1]
    sh = _shape(hq, hk, d, _dtype_code(qa))
    ru = _as_np(reused, np.uint8)
    outs = [np.empty((n,), np.float32) for _ in range(3)]
    rc = lib().kvso_first_order_impact(ctypes.byref(sh), ctypes.c_int64(n), _p(qa), _p(kf), _p(vf), _p(kc), _p(vc),
                                       _p(ru), ctypes.c_double(scale), _p(outs[0]), _p(outs[1]), _p(outs[2]))
    _check(rc, "first_order_impact")
    return tuple(outs)


def exact_impact(q, k_fresh, v_fresh, k_cache, v_cache, scale: float, reused=None) -> np.ndarray:
    """-> float32 [N]: the true L1 change of the attention output when token i alone is reused (tiny N only)."""
    qa = _as_np(q)
    kf, vf, kc, vc = _as_np(k_fresh), _as_np(v_fresh), _as_np(k_cache), _as_np(v_cache)
    n, hq, d = qa.shape
    hk = kf.shape[1]
    sh = _shape(hq, hk, d, _dtype_code(qa))
    ru = _as_np(reused, np.uint8)
    out = np.empty((n,), np.float32)
    rc = lib().kvso_exact_impact(ctypes.byref(sh), ctypes.c_int64(n), _p(qa), _p(kf), _p(vf), _p(kc), _p(vc),
                                 _p(ru), ctypes.c_double(scale), _p(out))
    _check(rc, "exact_impact")
    return out


def window_hash(tokens, window: int, base: int, modulus: int) -> np.ndarray:
    """App. E Eq. (7) for every window of ``window`` tokens: uint32 [n - window + 1]."""
    t = np.ascontiguousarray(np.asarray(tokens, dtype=np.int32))
    out = np.zeros((max(0, t.shape[0] - window + 1),), dtype=np.uint32)
    _check(lib().kvso_window_hash(_p(t), ctypes.c_int64(t.shape[0]), ctypes.c_int32(window), ctypes.c_uint32(base),
                                  ctypes.c_uint32(modulus), _p(out)), "window_hash")
    return out


def match_tokens(target, candidate, window: int, base: int, modulus: int):
    """App. E Alg. 3: (target_matches, candidate_matches) in the order of discovery, int32 each."""
    t = np.ascontiguousarray(np.asarray(target, dtype=np.int32))
    c = np.ascontiguousarray(np.asarray(candidate, dtype=np.int32))
    tm = np.zeros((max(1, t.shape[0]),), dtype=np.int32)
    cm = np.zeros((max(1, t.shape[0]),), dtype=np.int32)
    n = ctypes.c_int64(0)
    _check(lib().kvso_match_tokens(_p(t), ctypes.c_int64(t.shape[0]), _p(c), ctypes.c_int64(c.shape[0]),
                                   ctypes.c_int32(window), ctypes.c_uint32(base), ctypes.c_uint32(modulus),
                                   _p(tm), _p(cm), ctypes.byref(n)), "match_tokens")
    return tm[:n.value].copy(), cm[:n.value].copy()


def schedule(hit_rate) -> np.ndarray:
    """Sec. 4.3 Alg. 2: request indices in the queue's order (hit rate descending, arrival order among equals)."""
    h = np.ascontiguousarray(np.asarray(hit_rate, dtype=np.float32))
    order = np.zeros((h.shape[0],), dtype=np.int32)
    _check(lib().kvso_schedule(_p(h), ctypes.c_int32(h.shape[0]), _p(order)), "schedule")
    return order


def project_qkv(x, w, n_q_heads: int, n_kv_heads: int, head_dim: int, rows=None, pos=None, rope=None):
    """App. D.1: a layer's Q, K, V of the selected tokens (hidden states ``x`` [n_tokens, hidden], weight
    ``w`` [(n_q_heads + 2 n_kv_heads) head_dim, hidden]), rotary factors from ``rope`` [positions, head_dim/2, 2]
    applied to Q and K when given.  Returns fp64 arrays (q, k, v), unrounded."""
    xa, wa = _as_np(x), _as_np(w)
    code = _dtype_code(xa)
    if _dtype_code(wa) != code:
        raise TypeError("x and w must have one dtype")
    n_tokens, hidden = xa.shape
    ra = None if rows is None else np.ascontiguousarray(np.asarray(rows, dtype=np.int32))
    pa = None if pos is None else np.ascontiguousarray(np.asarray(pos, dtype=np.int32))
    n_sel = n_tokens if ra is None else ra.shape[0]
    rp = None if rope is None else np.ascontiguousarray(np.asarray(rope, dtype=np.float32))
    q = np.zeros((n_sel, n_q_heads, head_dim), dtype=np.float64)
    k = np.zeros((n_sel, n_kv_heads, head_dim), dtype=np.float64)
    v = np.zeros((n_sel, n_kv_heads, head_dim), dtype=np.float64)
    sh = _shape(n_q_heads, n_kv_heads, head_dim, code)
    _check(lib().kvso_project_qkv(ctypes.byref(sh), ctypes.c_int32(hidden), _p(xa), ctypes.c_int64(n_tokens), _p(ra), _p(pa),
                                  ctypes.c_int64(n_sel), _p(wa), _p(rp), ctypes.c_int64(0 if rp is None else rp.shape[0]),
                                  _p(q), _p(k), _p(v)), "project_qkv")
    return q, k, v


def decode_check(q_new, k_cache, dev_v, reused, scale: float, ctx_off, ctx_len, k_req,
                 v_cache=None, want_attn: bool = False):
    """-> (idx int32 packed, score float32 [rows] (nan where untouched), attn float64 or None)."""
    qa, ka = _as_np(q_new), _as_np(k_cache)
    va = _as_np(v_cache)
    b, hq, d = qa.shape
    rows, hk, _ = ka.shape
    dv = _as_np(dev_v, np.float32)
    ru = _as_np(reused, np.uint8)
    co = np.ascontiguousarray(np.asarray(ctx_off, dtype=np.int64))
    cl = np.ascontiguousarray(np.asarray(ctx_len, dtype=np.int64))
    kr = np.ascontiguousarray(np.asarray(k_req, dtype=np.int32))
    sh = _shape(hq, hk, d, _dtype_code(qa))
    idx = np.empty((int(kr.sum()),), np.int32)
    score = np.full((rows,), np.nan, np.float32)
    attn = np.empty((b, hq, d), np.float64) if want_attn else None
    rc = lib().kvso_decode_check(ctypes.byref(sh), ctypes.c_int32(b), ctypes.c_int64(rows), _p(co), _p(cl),
                                 _p(qa), _p(ka), _p(va), _p(dv), _p(ru), ctypes.c_double(scale),
                                 _p(kr), _p(idx), _p(score), _p(attn))
    _check(rc, "decode_check")
    return idx, score, attn
