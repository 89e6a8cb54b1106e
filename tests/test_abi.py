"""CPU-side checks of the C-ABI library: it loads without a GPU, exports every symbol the header
declares, and rejects bad arguments on the host before anything is launched (no compute calls
here: every call below fails validation or is a no-op by construction)."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2503_16525_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000  # non-NULL, 16-byte aligned, never dereferenced: validation fails first


@pytest.fixture(scope="module")
def lib():
    return B.load()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "kvs.h")).read()
    declared = re.findall(r"KVS_API\s+[\w\s\*]+?\b(kvs_\w+)\s*\(", header)
    assert sorted(declared) == sorted(B.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert lib.kvs_version().startswith(b"kvshare-hip gfx950")
    assert lib.kvs_strerror(B.EINVAL) == b"invalid argument"


def _shape(hq=32, hk=8, d=128, dt=B.BF16):
    return B.make_shape(hq, hk, d, dt)


def test_shape_validation(lib):
    for sh, want in [(_shape(hq=30), B.EINVAL), (_shape(d=96), B.EUNSUPPORTED), (_shape(dt=7), B.EINVAL),
                     (_shape(hk=0), B.EINVAL)]:
        rc = lib.kvs_deviation(ctypes.byref(sh), 16, None, FAKE, None, FAKE, None, None, 0, None, FAKE, FAKE, None)
        assert rc == want, lib.kvs_last_error()
    assert lib.kvs_deviation(None, 16, None, FAKE, None, FAKE, None, None, 0, None, FAKE, FAKE, None) == B.EINVAL


def test_deviation_argument_errors(lib):
    sh = _shape()
    assert lib.kvs_deviation(ctypes.byref(sh), -1, None, FAKE, None, FAKE, None, None, 0, None, None, None, None) == B.EINVAL
    assert lib.kvs_deviation(ctypes.byref(sh), 8, None, None, None, FAKE, None, None, 0, None, None, None, None) == B.EINVAL
    # mode KV needs the key tensors
    assert lib.kvs_deviation(ctypes.byref(sh), 8, None, FAKE, None, FAKE, None, None, 1, None, None, None, None) == B.EINVAL
    assert b"k_fresh" in lib.kvs_last_error()
    assert lib.kvs_deviation(ctypes.byref(sh), 8, None, FAKE + 4, None, FAKE, None, None, 0, None, None, None, None) == B.EINVAL
    assert lib.kvs_deviation(ctypes.byref(sh), 8, None, FAKE, None, FAKE, None, None, 5, None, None, None, None) == B.EINVAL
    # empty input: success, nothing launched
    assert lib.kvs_deviation(ctypes.byref(sh), 0, None, None, None, None, None, None, 0, None, None, None, None) == B.OK


def test_select_argument_errors(lib):
    ro = np.array([0, 10, 5], np.int64)
    kr = np.array([1, 1], np.int32)
    assert lib.kvs_select_topk(FAKE, 2, ro.ctypes.data, kr.ctypes.data, FAKE, None, 0, None) == B.EINVAL
    ro = np.array([0, 10], np.int64)
    for k in (-1, 11):
        kr = np.array([k], np.int32)
        assert lib.kvs_select_topk(FAKE, 1, ro.ctypes.data, kr.ctypes.data, FAKE, None, 0, None) == B.EINVAL
    kr = np.array([3], np.int32)
    assert lib.kvs_select_topk(None, 1, ro.ctypes.data, kr.ctypes.data, FAKE, None, 0, None) == B.EINVAL
    assert lib.kvs_select_topk(FAKE, -1, ro.ctypes.data, kr.ctypes.data, FAKE, None, 0, None) == B.EINVAL
    # the optional workspace must be 256-byte aligned; its size grows with the scores (one candidate slot each)
    assert lib.kvs_select_topk(FAKE, 1, ro.ctypes.data, kr.ctypes.data, FAKE, FAKE + 16, 4096, None) == B.EINVAL
    sh = _shape()
    small, large = B.kvs_workspace_size("select_topk", sh, 1, 1000), B.kvs_workspace_size("select_topk", sh, 4, 4 * 131072)
    assert 0 < small < large and large >= 4 * 4 * 131072
    # k = 0 everywhere and zero rows are no-ops
    kr = np.array([0], np.int32)
    assert lib.kvs_select_topk(None, 1, ro.ctypes.data, kr.ctypes.data, None, None, 0, None) == B.OK
    assert lib.kvs_select_topk(None, 0, None, None, None, None, 0, None) == B.OK


def test_scatter_argument_errors(lib):
    sh = _shape()
    assert lib.kvs_scatter_kv(ctypes.byref(sh), 100, FAKE, FAKE, FAKE, 101, FAKE, FAKE, None, None, None) == B.EINVAL
    assert lib.kvs_scatter_kv(ctypes.byref(sh), 100, None, FAKE, FAKE, 5, FAKE, FAKE, None, None, None) == B.EINVAL
    assert lib.kvs_scatter_kv(ctypes.byref(sh), 100, FAKE, FAKE, FAKE, -1, FAKE, FAKE, None, None, None) == B.EINVAL
    assert lib.kvs_scatter_kv(ctypes.byref(sh), 100, None, None, None, 0, None, None, None, None, None) == B.OK


def test_attention_argument_errors(lib):
    sh = _shape()
    co, cl = np.array([0], np.int64), np.array([100], np.int64)

    def call(cu, q=FAKE):
        cs = np.array(cu, np.int64)
        return lib.kvs_partial_attention(ctypes.byref(sh), 1, co.ctypes.data, cl.ctypes.data, cs.ctypes.data,
                                         q, FAKE, FAKE, FAKE, 1.0, FAKE, None, None, 0, None)
    assert call([0, 101]) == B.EINVAL          # more selected tokens than context rows
    assert call([1, 5]) == B.EINVAL            # cu_sel must start at 0
    assert call([0, 5], q=None) == B.EINVAL
    assert call([0, 5], q=FAKE + 2) == B.EINVAL
    assert call([0, 0], q=None) == B.OK        # nothing selected: no-op
    assert lib.kvs_partial_attention(ctypes.byref(sh), -1, None, None, None, None, None, None, None, 1.0,
                                     None, None, None, 0, None) == B.EINVAL


def test_decode_argument_errors(lib):
    sh = _shape()
    co, cl, kr = np.array([0, 50], np.int64), np.array([50, 60], np.int64), np.array([1, 1], np.int32)
    need = B.kvs_workspace_size("decode_check", sh, 2, 110)
    assert need >= 4 * 32 * 110

    def call(n_rows=110, ws=FAKE * 16, ws_bytes=need, k=kr, attn=None, v=None):
        return lib.kvs_decode_check(ctypes.byref(sh), 2, n_rows, co.ctypes.data, cl.ctypes.data, FAKE, FAKE, v,
                                    FAKE, None, 1.0, k.ctypes.data, FAKE, None, attn, ws, ws_bytes, None)
    assert call(n_rows=100) == B.EINVAL                       # second context overruns the cache
    assert call(ws_bytes=need - 1) == B.EWORKSPACE
    assert call(ws=None) == B.EWORKSPACE
    assert call(k=np.array([1, 61], np.int32)) == B.EINVAL
    assert call(attn=FAKE) == B.EINVAL                        # attn_out without v_cache
    assert b"v_cache" in lib.kvs_last_error()
    # contexts may not share cache rows, whichever order the requests come in
    for offs, lens in (([0, 40], [50, 60]), ([40, 0], [60, 50])):
        co2, cl2 = np.array(offs, np.int64), np.array(lens, np.int64)
        k0 = np.array([0, 0], np.int32)
        rc = lib.kvs_decode_check(ctypes.byref(sh), 2, 110, co2.ctypes.data, cl2.ctypes.data, FAKE, FAKE, None,
                                  FAKE, None, 1.0, k0.ctypes.data, FAKE, None, None, FAKE * 16, need, None)
        assert rc == B.EINVAL and b"cache rows" in lib.kvs_last_error()
    assert B.kvs_workspace_size("nonsense", sh, 1, 10) == 0


def test_attn_colsum_argument_errors(lib):
    sh = _shape()
    need = B.kvs_workspace_size("attn_colsum", sh, 1, 1000)
    assert need >= 4 * 32 * 1000

    def call(shape=sh, n=1000, q=FAKE, k=FAKE, scale=1.0, alpha=FAKE, ws=FAKE * 16, ws_bytes=need):
        return lib.kvs_attn_colsum(ctypes.byref(shape), n, q, k, scale, alpha, ws, ws_bytes, None)
    assert call(n=-1) == B.EINVAL
    assert call(n=0, q=None, k=None, alpha=None, ws=None, ws_bytes=0) == B.OK      # empty: no-op
    assert call(scale=float("nan")) == B.EINVAL
    assert call(q=None) == B.EINVAL
    assert call(k=FAKE + 8) == B.EINVAL
    assert call(ws=None) == B.EINVAL
    assert call(ws=FAKE * 16 + 64) == B.EINVAL                # workspace alignment
    assert call(ws_bytes=need - 1) == B.EWORKSPACE
    big = 1 << 20                                             # 8 GiB of queries: past the 32-bit offsets
    assert call(n=big, ws_bytes=B.kvs_workspace_size("attn_colsum", sh, 1, big)) == B.EUNSUPPORTED
    assert b"4 GiB" in lib.kvs_last_error()
    # shapes without a matrix-core kernel take the vector path, which refuses long contexts
    f32 = _shape(dt=B.F32, d=64, hq=4, hk=4)
    n_long = 1 << 17
    assert call(shape=f32, n=n_long, ws_bytes=B.kvs_workspace_size("attn_colsum", f32, 1, n_long)) == B.EUNSUPPORTED
    assert b"vector path" in lib.kvs_last_error()


def test_deviation_topk_argument_errors(lib):
    sh = _shape()

    def call(n=1000, k=10, idx=FAKE, ws=None, ws_bytes=0, v=FAKE):
        return lib.kvs_deviation_topk(ctypes.byref(sh), n, None, v, None, FAKE, None, None, 0, None, FAKE, FAKE,
                                      k, idx, ws, ws_bytes, None)
    assert call(n=-1) == B.EINVAL
    assert call(k=-1) == B.EINVAL
    assert call(k=1001) == B.EINVAL and b"outside" in lib.kvs_last_error()
    assert call(idx=None) == B.EINVAL
    assert call(ws=FAKE * 16 + 64, ws_bytes=1 << 20) == B.EINVAL          # workspace alignment
    assert call(v=None) == B.EINVAL                                        # the scoring call's own checks still apply
    assert call(n=0, k=0, idx=None, v=None) == B.OK                        # empty: no-op


def test_first_order_impact_argument_errors(lib):
    sh = _shape()
    need = B.kvs_workspace_size("first_order_impact", sh, 1, 500)
    assert need >= 3 * 4 * 8 * 500

    def call(n=500, q=FAKE, lse=FAKE, scale=1.0, ws=FAKE * 16, ws_bytes=need):
        return lib.kvs_first_order_impact(ctypes.byref(sh), n, q, FAKE, FAKE, FAKE, FAKE, FAKE, lse, None, scale,
                                          FAKE, FAKE, FAKE, ws, ws_bytes, None)
    assert call(n=-1) == B.EINVAL
    assert call(n=0) == B.OK                                               # empty: no-op
    assert call(n=(1 << 20) + 1, ws_bytes=1 << 40) == B.EUNSUPPORTED
    assert call(q=None) == B.EINVAL
    assert call(lse=None) == B.EINVAL
    assert call(scale=float("inf")) == B.EINVAL
    assert call(ws=None) == B.EWORKSPACE
    assert call(ws_bytes=need - 1) == B.EWORKSPACE
    assert call(ws=FAKE * 16 + 64) == B.EINVAL


def test_match_tokens_argument_errors(lib):
    need = B.kvs_workspace_size("match_tokens", None, 1, 4000, 3000)
    assert need > 0

    def call(nt=4000, nc=3000, w=16, m=4294967291, targ=FAKE, cand=FAKE, partner=FAKE, n_out=FAKE, ws=FAKE * 16, ws_bytes=need):
        return lib.kvs_match_tokens(targ, nt, cand, nc, w, 1000003, m, partner, None, None, n_out, ws, ws_bytes, None)
    assert call(nt=-1) == B.EINVAL
    assert call(nc=-1) == B.EINVAL
    assert call(w=0) == B.EINVAL
    assert call(m=0) == B.EINVAL and b"modulus" in lib.kvs_last_error()
    assert call(nt=(1 << 26) + 1) == B.EUNSUPPORTED
    assert call(n_out=None) == B.EINVAL
    assert call(targ=None) == B.EINVAL
    assert call(partner=None) == B.EINVAL
    assert call(cand=None) == B.EINVAL
    assert call(ws=None) == B.EINVAL
    assert call(ws=FAKE * 16 + 64) == B.EINVAL
    assert call(ws_bytes=need - 1) == B.EWORKSPACE
    # the workspace grows with both sequences
    assert B.kvs_workspace_size("match_tokens", None, 1, 8000, 3000) > need
    assert B.kvs_workspace_size("match_tokens", None, 1, 4000, 6000) > need


def test_project_qkv_argument_errors(lib):
    sh = _shape()

    def call(shape=sh, hidden=4096, x=FAKE, n_tok=1000, rows=None, pos=FAKE, n_sel=100, wq=FAKE, rope=FAKE, rope_n=2048,
             q=FAKE, k=FAKE, v=FAKE):
        return lib.kvs_project_qkv(ctypes.byref(shape), hidden, x, n_tok, rows, pos, n_sel, wq, rope, rope_n, q, k, v, None)
    assert call(n_tok=-1) == B.EINVAL
    assert call(n_sel=-1) == B.EINVAL
    assert call(shape=_shape(dt=B.F32, d=64, hq=4, hk=4)) == B.EUNSUPPORTED
    assert call(shape=_shape(hq=3, hk=1)) == B.EUNSUPPORTED               # 5 heads in all: odd
    assert call(hidden=4096 + 32) == B.EUNSUPPORTED
    assert call(hidden=0) == B.EUNSUPPORTED
    assert call(n_sel=0, x=None, wq=None, q=None, k=None, v=None) == B.OK  # nothing selected: no-op
    assert call(n_tok=0) == B.EINVAL
    assert call(n_sel=1001) == B.EINVAL                                    # without a row list the first n_sel rows of x are meant
    assert call(x=None) == B.EINVAL
    assert call(v=None) == B.EINVAL
    assert call(pos=None) == B.EINVAL and b"rotary" in lib.kvs_last_error()
    assert call(rope_n=0) == B.EINVAL
    assert call(wq=FAKE + 8) == B.EINVAL
    assert call(n_tok=1 << 20) == B.EUNSUPPORTED and b"4 GiB" in lib.kvs_last_error()
    assert call(rope_n=1 << 23) == B.EUNSUPPORTED and b"rotary" in lib.kvs_last_error()
