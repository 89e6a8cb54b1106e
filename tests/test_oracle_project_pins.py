"""Pins for the oracle's selected-token projection (App. D.1: the tokens picked in an early layer are the
ones recomputed later; recomputing a token's Q/K/V in a layer is that layer's projection of its hidden state,
with the rotary position factors of the evaluated model families on Q and K).

Pinned by numpy's matrix product, by the rotation written as a complex multiplication, by a quarter turn
worked by hand, and by what a rotation must preserve (norms, position 0, relative positions)."""
import numpy as np
import torch

import oracle
from paper_2503_16525_amd import synth


def test_projection_is_a_matrix_product_split_by_heads():
    rng = np.random.default_rng(0)
    hq, hk, d, hidden, n = 4, 2, 8, 24, 11
    x = rng.standard_normal((n, hidden)).astype(np.float32)
    w = rng.standard_normal(((hq + 2 * hk) * d, hidden)).astype(np.float32)
    rows = np.array([7, 0, 10, 3, 3], dtype=np.int32)
    q, k, v = oracle.project_qkv(x, w, hq, hk, d, rows=rows)
    y = x[rows].astype(np.float64) @ w.astype(np.float64).T
    np.testing.assert_allclose(q.reshape(5, -1), y[:, :hq * d], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(k.reshape(5, -1), y[:, hq * d:(hq + hk) * d], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(v.reshape(5, -1), y[:, (hq + hk) * d:], rtol=1e-13, atol=1e-13)
    # no row list = every token in order
    q2, _, _ = oracle.project_qkv(x, w, hq, hk, d)
    q3, _, _ = oracle.project_qkv(x, w, hq, hk, d, rows=np.arange(n))
    assert np.array_equal(q2, q3)


def test_bf16_inputs_widen_exactly():
    gen = torch.Generator().manual_seed(1)
    x = torch.randn((6, 16), generator=gen).to(torch.bfloat16)
    w = torch.randn((3 * 4, 16), generator=gen).to(torch.bfloat16)
    q, k, v = oracle.project_qkv(x, w, 1, 1, 4)
    y = x.double().numpy() @ w.double().numpy().T
    np.testing.assert_allclose(np.concatenate([q, k, v], axis=1).reshape(6, -1), y, rtol=1e-13, atol=1e-13)


def test_quarter_turn_by_hand():
    # one head of two channels, identity projection; the table turns position 1 by 90 degrees:
    # (a, b) -> (a cos - b sin, b cos + a sin) = (-b, a)
    x = np.array([[3.0, 4.0], [3.0, 4.0]], dtype=np.float32)
    w = np.concatenate([np.eye(2), np.eye(2), np.eye(2)]).astype(np.float32)
    rope = np.array([[[1.0, 0.0]], [[0.0, 1.0]]], dtype=np.float32)       # [2 positions, 1 pair, (cos, sin)]
    q, k, v = oracle.project_qkv(x, w, 1, 1, 2, pos=[0, 1], rope=rope)
    assert q[0, 0].tolist() == [3.0, 4.0] and q[1, 0].tolist() == [-4.0, 3.0]
    assert k[1, 0].tolist() == [-4.0, 3.0]
    assert v[1, 0].tolist() == [3.0, 4.0]                                   # V is not turned


def test_rotation_as_complex_multiplication_and_invariants():
    rng = np.random.default_rng(3)
    hq, hk, d, hidden, n = 6, 2, 16, 40, 9
    x = rng.standard_normal((n, hidden)).astype(np.float32)
    w = rng.standard_normal(((hq + 2 * hk) * d, hidden)).astype(np.float32)
    rope = synth.make_rope_table(500, d, theta=10000.0)
    pos = rng.integers(0, 500, size=n).astype(np.int32)
    q, k, v = oracle.project_qkv(x, w, hq, hk, d, pos=pos, rope=rope)
    q0, k0, v0 = oracle.project_qkv(x, w, hq, hk, d)
    turn = (rope[pos, :, 0].astype(np.float64) + 1j * rope[pos, :, 1].astype(np.float64))[:, None, :]     # [n, 1, d/2]
    for got, plain in ((q, q0), (k, k0)):
        z = (plain[..., :d // 2] + 1j * plain[..., d // 2:]) * turn
        np.testing.assert_allclose(got[..., :d // 2], z.real, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(got[..., d // 2:], z.imag, rtol=1e-12, atol=1e-12)
        # a rotation keeps the length of every channel pair (the table's fp32 rounding: 1e-7)
        np.testing.assert_allclose(got[..., :d // 2] ** 2 + got[..., d // 2:] ** 2,
                                   plain[..., :d // 2] ** 2 + plain[..., d // 2:] ** 2, rtol=1e-6)
    assert np.array_equal(v, v0)
    # position 0 turns nothing
    qz, kz, _ = oracle.project_qkv(x, w, hq, hk, d, pos=np.zeros(n, dtype=np.int32), rope=rope)
    assert np.array_equal(qz, q0) and np.array_equal(kz, k0)
    # scores depend on the difference of the positions only
    qa, ka, _ = oracle.project_qkv(x[:2], w, hq, hk, d, pos=[40, 7], rope=rope)
    qb, kb, _ = oracle.project_qkv(x[:2], w, hq, hk, d, pos=[140, 107], rope=rope)
    sa = np.einsum("hc,c->h", qa[0], ka[1, 0])
    sb = np.einsum("hc,c->h", qb[0], kb[1, 0])
    np.testing.assert_allclose(sa, sb, rtol=1e-5, atol=1e-5)


def test_rope_table_generator():
    t = synth.make_rope_table(8, 4, theta=100.0)
    assert t.shape == (8, 2, 2)
    np.testing.assert_allclose(t[3, 0], [np.cos(3.0), np.sin(3.0)], rtol=1e-7)          # frequency 0: one radian per position
    np.testing.assert_allclose(t[3, 1], [np.cos(0.3), np.sin(0.3)], rtol=1e-7)          # frequency 1: theta^(-1/2) = 0.1
