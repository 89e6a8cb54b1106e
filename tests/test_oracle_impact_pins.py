"""Pins for the oracle's first-order impact scores (Sec. 4.1, Eq. (2)) and the exact single-token
impact (the "ideal index" of Sec. 4.1 / App. D.2).  CPU only.

What fixes them from outside: the Jacobian-vector product of a library autodiff on the textbook
attention (the hand-derived softmax Jacobian against torch.autograd), finite differences of the
exact impact (first order is the limit of true change / step), and the two special cases the
paper states: with no key deviation the movement is A dV exactly (dH/dV = A), which ties the
value-direction impact to the column mass alpha and to Eq. (3); with no value deviation only the
key term is left."""
import math

import numpy as np
import pytest
import torch

import oracle


def _case(n=20, hq=4, hk=2, d=8, seed=0, eps_k=0.05, eps_v=0.05, dtype=torch.float32):
    g = torch.Generator().manual_seed(seed)
    q = (torch.randn((n, hq, d), generator=g) / math.sqrt(d) * 2.0).to(dtype)
    kf = torch.randn((n, hk, d), generator=g).to(dtype)
    vf = torch.randn((n, hk, d), generator=g).to(dtype)
    kc = (kf.float() + eps_k * torch.randn((n, hk, d), generator=g)).to(dtype)
    vc = (vf.float() + eps_v * torch.randn((n, hk, d), generator=g)).to(dtype)
    return q, kf, vf, kc, vc


def _attention_all_heads(q, k, v, scale):
    """textbook causal attention in fp64 with torch ops: q [n,hq,d], k/v [n,hk,d] -> [hq,n,d]"""
    n, hq, d = q.shape
    hk = k.shape[1]
    grp = hq // hk
    kk = k.repeat_interleave(grp, dim=1)      # head h reads kv head h // grp
    vv = v.repeat_interleave(grp, dim=1)
    s = torch.einsum("jhc,ihc->hji", q, kk) * scale
    mask = torch.tril(torch.ones(n, n, dtype=torch.bool))
    s = s.masked_fill(~mask, float("-inf"))
    return torch.einsum("hji,ihc->hjc", torch.softmax(s, dim=-1), vv)


@pytest.mark.parametrize("hq,hk", [(2, 2), (4, 2), (6, 2)])
def test_first_order_terms_are_the_autodiff_jacobian_vector_products(hq, hk):
    q, kf, vf, kc, vc = _case(n=14, hq=hq, hk=hk, d=8, seed=3)
    scale = 0.7
    imp_v, imp_k, imp_kv = oracle.first_order_impact(q, kf, vf, kc, vc, scale)
    qd, kd, vd = q.double(), kf.double(), vf.double()
    dk, dv = kc.double() - kd, vc.double() - vd
    for i in (0, 5, 13):
        tk, tv = torch.zeros_like(kd), torch.zeros_like(vd)
        tk[i], tv[i] = dk[i], dv[i]              # only token i deviates
        f = lambda k_, v_: _attention_all_heads(qd, k_, v_, scale)
        _, j_kv = torch.autograd.functional.jvp(f, (kd, vd), (tk, tv))
        _, j_k = torch.autograd.functional.jvp(f, (kd, vd), (tk, torch.zeros_like(vd)))
        _, j_v = torch.autograd.functional.jvp(f, (kd, vd), (torch.zeros_like(kd), tv))
        np.testing.assert_allclose(imp_kv[i], j_kv.abs().sum().item(), rtol=2e-6)
        np.testing.assert_allclose(imp_k[i], j_k.abs().sum().item(), rtol=2e-6)
        np.testing.assert_allclose(imp_v[i], j_v.abs().sum().item(), rtol=2e-6)


def test_first_order_is_the_limit_of_the_exact_impact():
    """exact change / first-order prediction -> 1 as the deviation shrinks, with an error that
    shrinks in proportion (second-order remainder)."""
    gaps = []
    for eps in (2.0 ** -6, 2.0 ** -9):
        q, kf, vf, kc, vc = _case(n=16, hq=4, hk=2, d=8, seed=5, eps_k=eps, eps_v=eps)
        _, _, first = oracle.first_order_impact(q, kf, vf, kc, vc, 1.0)
        exact = oracle.exact_impact(q, kf, vf, kc, vc, 1.0)
        gaps.append(np.max(np.abs(exact / first - 1.0)))
    assert gaps[0] < 0.05 and gaps[1] < 0.01
    assert gaps[1] < gaps[0] / 4          # eight times smaller step: the gap falls about as much


def test_without_key_deviation_the_impact_is_alpha_times_the_value_deviation():
    """dK = 0: H' - H = A dV exactly (Sec. 4.1: dH/dV = A), so the exact impact, the first-order one and
    Eq. (3)'s score -- column mass times the L1 norm of dV, per head group -- are one number."""
    q, kf, vf, _, vc = _case(n=24, hq=6, hk=3, d=8, seed=7)
    reused = (np.arange(24) % 3 != 0).astype(np.uint8)
    imp_v, imp_k, imp_kv = oracle.first_order_impact(q, kf, vf, kf, vc, 0.9, reused=reused)
    exact = oracle.exact_impact(q, kf, vf, kf, vc, 0.9, reused=reused)
    _, alpha_g = oracle.alpha_prefill(q, kf, 0.9)
    _, _, score = oracle.deviation(vf, vc, reused=reused, alpha=alpha_g.astype(np.float32))
    cand = reused != 0
    assert np.all(np.isneginf(imp_v[~cand])) and np.all(np.isneginf(imp_kv[~cand])) and np.all(np.isneginf(exact[~cand]))
    assert np.all(imp_k[cand] == 0)
    np.testing.assert_allclose(imp_kv[cand], imp_v[cand], rtol=1e-6)
    np.testing.assert_allclose(exact[cand], imp_v[cand], rtol=1e-5)
    np.testing.assert_allclose(score[cand], imp_v[cand], rtol=1e-5)       # Eq. (3) through kvso_deviation + kvso_alpha_prefill


def test_without_value_deviation_only_the_key_term_is_left():
    q, kf, vf, kc, _ = _case(n=18, hq=2, hk=1, d=16, seed=9)
    imp_v, imp_k, imp_kv = oracle.first_order_impact(q, kf, vf, kc, vf, 1.0)
    assert np.all(imp_v == 0) and np.all(imp_k > 0)
    np.testing.assert_array_equal(imp_kv, imp_k)
    # the last token is only seen by its own row, where the key term is a (1 - a)-weighted shift
    # towards its own value: a one-row closed form
    n = 18
    qd, kd, vd = q.double()[n - 1, :, :], kf.double()[:, 0, :], vf.double()[:, 0, :]
    dk = (kc.double() - kf.double())[n - 1, 0]
    want = 0.0
    for h in range(2):
        s = kd @ qd[h]
        a = torch.softmax(s, dim=0)
        hrow = a @ vd
        want += (a[n - 1] * torch.dot(qd[h], dk) * (vd[n - 1] - hrow)).abs().sum().item()
    np.testing.assert_allclose(imp_k[n - 1], want, rtol=1e-6)


def test_impact_on_bf16_inputs_widens_exactly():
    """bf16 bit patterns are widened exactly: the same numbers given as fp32 give the same impacts."""
    q, kf, vf, kc, vc = _case(n=12, hq=4, hk=2, d=8, seed=11, dtype=torch.bfloat16)
    a = oracle.first_order_impact(q, kf, vf, kc, vc, 1.0)
    b = oracle.first_order_impact(q.float(), kf.float(), vf.float(), kc.float(), vc.float(), 1.0)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)
    np.testing.assert_array_equal(oracle.exact_impact(q, kf, vf, kc, vc, 1.0),
                                  oracle.exact_impact(q.float(), kf.float(), vf.float(), kc.float(), vc.float(), 1.0))
