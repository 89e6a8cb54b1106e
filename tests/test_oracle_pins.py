"""Pins for the CPU oracle: every oracle function is checked against something other than
itself -- a library routine on a special case, a closed form, an invariant, or brute force on
tiny inputs -- chosen so that a dropped term, a wrong sign/index or a transposed operand fails.

No GPU needed.  The paper prints no worked numeric example of Alg. 1, so there are no printed
values to match; the pins below are what the paper's formulas and the mathematics fix.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2503_16525_amd import synth

torch.manual_seed(0)


def _rand(shape, dtype=torch.float32, seed=0, std=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * std).to(dtype)


# ------------------------------------------------------------------------------- O1 deviation

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_deviation_is_l1_norm_library(dtype):
    # Eq. (3): ||Delta V_i||_1 -- numpy's 1-norm on the same bits, per (token, kv head)
    n, hk, d = 37, 3, 16
    vf, vc = _rand((n, hk, d), dtype, 1), _rand((n, hk, d), dtype, 2)
    kf, kc = _rand((n, hk, d), dtype, 3), _rand((n, hk, d), dtype, 4)
    dev_k, dev_v, score = oracle.deviation(vf, vc, kf, kc, mode=oracle.SCORE_KV)
    ref_v = np.linalg.norm((vf.double() - vc.double()).numpy(), ord=1, axis=-1).T  # [hk, n]
    ref_k = np.linalg.norm((kf.double() - kc.double()).numpy(), ord=1, axis=-1).T
    np.testing.assert_allclose(dev_v, ref_v.astype(np.float32), rtol=0, atol=0)
    np.testing.assert_allclose(dev_k, ref_k.astype(np.float32), rtol=0, atol=0)
    np.testing.assert_allclose(score, (ref_v + ref_k).sum(0), rtol=1e-6)


def test_deviation_special_cases_and_indexing():
    n, hk, d = 11, 4, 8
    vf = _rand((n, hk, d), torch.float32, 5)
    _, dev_v, score = oracle.deviation(vf, vf.clone())
    assert np.all(dev_v == 0) and np.all(score == 0)
    # one perturbed element lands in exactly one (head, token) cell with its magnitude
    vc = vf.clone()
    vc[7, 2, 5] += 0.375
    _, dev_v, score = oracle.deviation(vf, vc)
    expect = np.zeros((hk, n), np.float32)
    expect[2, 7] = 0.375
    np.testing.assert_allclose(dev_v, expect, atol=1e-7)
    assert score[7] == pytest.approx(0.375, abs=1e-7) and np.count_nonzero(score) == 1
    # sign of the difference is irrelevant
    vc2 = vf.clone()
    vc2[7, 2, 5] -= 0.375
    np.testing.assert_allclose(oracle.deviation(vf, vc2)[1], expect, atol=1e-7)


def test_deviation_statistical_closed_form():
    # cache = fresh + sigma_i * N(0,1)  =>  E ||dV||_1 = d * sigma_i * sqrt(2/pi)
    lay = synth.make_layer(synth.TINY)
    _, dev_v, _ = oracle.deviation(lay["v_fresh"], lay["v_cache"])
    m = lay["reused"].numpy().astype(bool)
    sig = lay["sigma"].numpy()
    ratio = dev_v[:, m].mean(0) / (synth.TINY.head_dim * sig[m] * math.sqrt(2 / math.pi))
    assert abs(ratio.mean() - 1.0) < 0.02
    assert np.all(dev_v[:, ~m] == 0)


# ------------------------------------------------------------------------------- O3 score

def test_score_weighting_mask_and_linearity():
    n, hk, d = 29, 3, 8
    vf, vc = _rand((n, hk, d), torch.float32, 6), _rand((n, hk, d), torch.float32, 7)
    reused = (torch.arange(n) % 3 != 0).to(torch.uint8)
    alpha = torch.rand((hk, n), generator=torch.Generator().manual_seed(8)) + 0.1
    _, dev_v, s1 = oracle.deviation(vf, vc, reused=reused)
    # alpha == 1  =>  sum over heads of the L1 norms; -inf exactly off the candidate set
    m = reused.numpy().astype(bool)
    np.testing.assert_allclose(s1[m], dev_v.sum(0)[m], rtol=1e-6)
    assert np.all(np.isneginf(s1[~m])) and np.all(np.isfinite(s1[m]))
    # weighted: library dot product over heads; linear in alpha
    _, _, sa = oracle.deviation(vf, vc, reused=reused, alpha=alpha)
    ref = np.einsum("gn,gn->n", alpha.double().numpy(), dev_v.astype(np.float64))
    np.testing.assert_allclose(sa[m], ref[m], rtol=1e-6)
    _, _, s2a = oracle.deviation(vf, vc, reused=reused, alpha=2 * alpha)
    np.testing.assert_allclose(s2a[m], 2 * sa[m], rtol=1e-6)
    # a one-hot alpha picks out one head's deviation (catches a head/token transposition)
    onehot = torch.zeros((hk, n))
    onehot[1] = 1.0
    _, _, s_h = oracle.deviation(vf, vc, alpha=onehot)
    np.testing.assert_allclose(s_h, dev_v[1], rtol=1e-6)


def test_score_two_token_closed_form():
    # N=2, one head, d=1.  Row 0 attends only to token 0; row 1 splits by a logistic:
    # alpha_0 = 1 + sigmoid(scale*q1*(k0-k1)), alpha_1 = 1 - sigmoid(...).   Eq. (3) then gives
    # Score_i = alpha_i * |dv_i|.
    q = torch.tensor([[[0.3]], [[-1.25]]])
    k = torch.tensor([[[0.5]], [[2.0]]])
    scale = 0.7
    ah, ag = oracle.alpha_prefill(q, k, scale)
    sg = 1.0 / (1.0 + math.exp(-scale * (-1.25) * (0.5 - 2.0)))
    np.testing.assert_allclose(ah[0], [1 + sg, 1 - sg], rtol=1e-12)
    vf = torch.tensor([[[1.0]], [[-2.0]]])
    vc = torch.tensor([[[1.5]], [[-2.25]]])
    _, _, score = oracle.deviation(vf, vc, alpha=torch.from_numpy(ag).float())
    np.testing.assert_allclose(score, [(1 + sg) * 0.5, (1 - sg) * 0.25], rtol=1e-6)


# ------------------------------------------------------------------------------- O2 alpha

def _dense_causal_probs(q, k, scale):
    """[Hq, N, N] float64 causal softmax with torch library ops (GQA by repeat_interleave)."""
    n, hq, d = q.shape
    hk = k.shape[1]
    kk = k.double().repeat_interleave(hq // hk, dim=1)            # [N, Hq, d]
    logits = torch.einsum("jhd,ihd->hji", q.double(), kk) * scale
    mask = torch.tril(torch.ones(n, n, dtype=torch.bool))
    logits = logits.masked_fill(~mask, float("-inf"))
    return torch.softmax(logits, dim=-1)


@pytest.mark.parametrize("dtype,hq,hk", [(torch.float32, 4, 4), (torch.bfloat16, 6, 2), (torch.float32, 7, 1)])
def test_alpha_matches_dense_softmax_colsum(dtype, hq, hk):
    n, d = 96, 16
    q, k = _rand((n, hq, d), dtype, 11, 0.5), _rand((n, hk, d), dtype, 12)
    scale = 0.9
    ah, ag = oracle.alpha_prefill(q, k, scale)
    probs = _dense_causal_probs(q, k, scale)
    np.testing.assert_allclose(ah, probs.sum(1).numpy(), rtol=1e-10)
    grp = hq // hk
    np.testing.assert_allclose(ag, probs.sum(1).view(hk, grp, n).sum(1).numpy(), rtol=1e-10)


def test_alpha_invariants_and_harmonic_closed_form():
    n, hq, hk, d = 200, 4, 2, 8
    q, k = _rand((n, hq, d), torch.float32, 13), _rand((n, hk, d), torch.float32, 14)
    ah, ag = oracle.alpha_prefill(q, k, 1.0 / math.sqrt(d))
    np.testing.assert_allclose(ah.sum(1), n, rtol=1e-12)       # every row of A sums to 1
    assert np.all(ah[:, 0] >= 1.0) and np.all(ah[:, -1] <= 1.0) and np.all(ah > 0)
    np.testing.assert_allclose(ag.sum(), n * hq, rtol=1e-12)
    # Q == 0: uniform causal rows, alpha_i = sum_{j>=i} 1/(j+1)
    ah0, _ = oracle.alpha_prefill(torch.zeros_like(q), k, 1.0)
    inv = 1.0 / np.arange(1, n + 1)
    tail = np.cumsum(inv[::-1])[::-1]
    np.testing.assert_allclose(ah0, np.broadcast_to(tail, (hq, n)), rtol=1e-12)


# ------------------------------------------------------------------------------- O4 select

def _brute_select(row, k):
    order = sorted(range(len(row)), key=lambda i: (-float(row[i]), i))
    return np.array(sorted(order[:k]), dtype=np.int32)


def test_select_brute_force_random_and_ties():
    rng = np.random.default_rng(3)
    rows, ks = [], []
    for t in range(40):
        n = int(rng.integers(1, 400))
        r = rng.standard_normal(n).astype(np.float32)
        if t % 2:                       # heavy ties: quantise to a few levels
            r = np.round(r * 2) / 2
        if t % 5 == 0:
            r[rng.random(n) < 0.3] = -np.inf
        rows.append(r)
        ks.append(int(rng.integers(0, n + 1)))
    off = np.concatenate([[0], np.cumsum([len(r) for r in rows])])
    got = oracle.select_topk(np.concatenate(rows), off, ks)
    pos = 0
    for r, k in zip(rows, ks):
        np.testing.assert_array_equal(got[pos:pos + k], _brute_select(r, k))
        pos += k
    assert pos == len(got)


def test_select_edge_cases():
    s = np.array([1.0, 3.0, 3.0, -np.inf, 0.0, -0.0, 3.0, 2.0], np.float32)
    n = len(s)
    assert len(oracle.select_topk(s, [0, n], [0])) == 0
    np.testing.assert_array_equal(oracle.select_topk(s, [0, n], [n]), np.arange(n))
    np.testing.assert_array_equal(oracle.select_topk(s, [0, n], [2]), [1, 2])       # lowest indices of the tie
    np.testing.assert_array_equal(oracle.select_topk(s, [0, n], [4]), [1, 2, 6, 7])
    np.testing.assert_array_equal(oracle.select_topk(s, [0, n], [6]), [0, 1, 2, 4, 6, 7])  # +0 before -0 by index
    np.testing.assert_array_equal(oracle.select_topk(s, [0, n], [7]), [0, 1, 2, 4, 5, 6, 7])
    np.testing.assert_array_equal(oracle.select_topk(np.full(9, 2.5, np.float32), [0, 9], [4]), [0, 1, 2, 3])
    with pytest.raises(ValueError):
        oracle.select_topk(np.array([1.0, np.nan], np.float32), [0, 2], [1])
    with pytest.raises(ValueError):
        oracle.select_topk(s, [0, n], [n + 1])
    # two rows: the second row's indices are row-local
    got = oracle.select_topk(s, [0, 4, 8], [1, 2])
    np.testing.assert_array_equal(got, [1, 2, 3])


def test_select_invariants_large():
    rng = np.random.default_rng(9)
    n, k = 5000, 617
    s = rng.lognormal(-3, 1.5, n).astype(np.float32)
    s[rng.random(n) < 0.1] = -np.inf
    idx = oracle.select_topk(s, [0, n], [k])
    assert len(idx) == k and np.all(np.diff(idx) > 0)
    chosen = np.zeros(n, bool)
    chosen[idx] = True
    assert s[chosen].min() >= s[~chosen].max()
    # numpy's stable argsort on the negated scores is the same order
    np.testing.assert_array_equal(idx, np.sort(np.argsort(-s, kind="stable")[:k]))


# ------------------------------------------------------------------------------- O5 scatter

def test_scatter_is_indexed_assignment():
    n, hk, d, ns = 50, 2, 8, 9
    for dtype in (torch.float32, torch.bfloat16):
        kc, vc = _rand((n, hk, d), dtype, 20), _rand((n, hk, d), dtype, 21)
        kn, vn = _rand((ns, hk, d), dtype, 22), _rand((ns, hk, d), dtype, 23)
        pos = torch.tensor([3, 4, 10, 11, 12, 30, 31, 48, 49], dtype=torch.int32)
        k_np, v_np = oracle._as_np(kc).copy(), oracle._as_np(vc).copy()
        reused = np.ones(n, np.uint8)
        dev = np.ones((hk, n), np.float32)
        oracle.scatter_kv(kn, vn, pos, k_np, v_np, reused, dev)
        k_ref, v_ref = kc.clone(), vc.clone()
        k_ref[pos.long()] = kn
        v_ref[pos.long()] = vn
        np.testing.assert_array_equal(k_np, oracle._as_np(k_ref))
        np.testing.assert_array_equal(v_np, oracle._as_np(v_ref))
        exp_r = np.ones(n, np.uint8)
        exp_r[pos.numpy()] = 0
        np.testing.assert_array_equal(reused, exp_r)
        np.testing.assert_array_equal(dev, np.broadcast_to(exp_r.astype(np.float32), (hk, n)))


# ------------------------------------------------------------------------------- O6 attention

def _sdpa_causal(q, k, v, scale):
    """Library routine: torch scaled_dot_product_attention, float64, causal, GQA expanded."""
    n, hq, d = q.shape
    hk = k.shape[1]
    qq = q.double().permute(1, 0, 2).unsqueeze(0)
    kk = k.double().repeat_interleave(hq // hk, dim=1).permute(1, 0, 2).unsqueeze(0)
    vv = v.double().repeat_interleave(hq // hk, dim=1).permute(1, 0, 2).unsqueeze(0)
    o = torch.nn.functional.scaled_dot_product_attention(qq, kk, vv, is_causal=True, scale=scale)
    return o[0].permute(1, 0, 2).numpy()


@pytest.mark.parametrize("dtype,hq,hk,d", [(torch.float32, 4, 4, 16), (torch.bfloat16, 8, 2, 32),
                                           (torch.float32, 7, 1, 8)])
def test_attention_all_rows_is_causal_sdpa(dtype, hq, hk, d):
    n = 70
    q, k, v = _rand((n, hq, d), dtype, 30, 0.6), _rand((n, hk, d), dtype, 31), _rand((n, hk, d), dtype, 32)
    scale = 1.0 / math.sqrt(d)
    out, lse = oracle.partial_attention(q, np.arange(n, dtype=np.int32), k, v, scale)
    np.testing.assert_allclose(out, _sdpa_causal(q, k, v, scale), rtol=1e-10, atol=1e-12)
    kk = k.double().repeat_interleave(hq // hk, dim=1)
    logits = torch.einsum("jhd,ihd->jhi", q.double(), kk) * scale
    logits = logits.masked_fill(~torch.tril(torch.ones(n, n, dtype=torch.bool)).unsqueeze(1), float("-inf"))
    np.testing.assert_allclose(lse, torch.logsumexp(logits, -1).numpy(), rtol=1e-10)


def test_attention_subset_rows_and_special_cases():
    n, hq, hk, d = 90, 6, 3, 16
    q, k, v = _rand((n, hq, d), torch.float32, 33), _rand((n, hk, d), torch.float32, 34), _rand((n, hk, d), torch.float32, 35)
    scale = 0.31
    full = _sdpa_causal(q, k, v, scale)
    pos = np.array([0, 5, 6, 40, 89], np.int32)
    out, _ = oracle.partial_attention(q[pos.astype(np.int64)], pos, k, v, scale)
    np.testing.assert_allclose(out, full[pos], rtol=1e-10, atol=1e-12)
    # p = 0 attends to token 0 alone
    np.testing.assert_allclose(out[0], v[0].double().repeat_interleave(hq // hk, 0).numpy(), rtol=1e-12)
    # constant V -> that constant
    vc = torch.full_like(v, 0.75)
    outc, _ = oracle.partial_attention(q[pos.astype(np.int64)], pos, k, vc, scale)
    np.testing.assert_allclose(outc, 0.75, rtol=1e-12)
    # heads of one group with the same query give the same output
    qs = q[pos.astype(np.int64)].clone()
    qs[:, 1] = qs[:, 0]
    outg, _ = oracle.partial_attention(qs, pos, k, v, scale)
    np.testing.assert_array_equal(outg[:, 0], outg[:, 1])
    assert not np.allclose(outg[:, 0], outg[:, 2])


def test_attention_ragged_batch_equals_per_request():
    hq, hk, d = 4, 2, 8
    lens = [33, 1, 50]
    pad = 3                                    # slack rows between requests
    off = np.cumsum([0] + [l + pad for l in lens])[:-1]
    rows = sum(lens) + pad * len(lens)
    k, v = _rand((rows, hk, d), torch.bfloat16, 36), _rand((rows, hk, d), torch.bfloat16, 37)
    sel = [np.array([2, 10, 32], np.int32), np.array([0], np.int32), np.array([], np.int32)]
    cu = np.cumsum([0] + [len(s) for s in sel])
    q = _rand((int(cu[-1]), hq, d), torch.bfloat16, 38)
    out, lse = oracle.partial_attention(q, np.concatenate(sel), k, v, 0.4, off, lens, cu)
    for b in range(3):
        if len(sel[b]) == 0:
            continue
        sl = slice(int(off[b]), int(off[b]) + lens[b])
        ob, lb = oracle.partial_attention(q[cu[b]:cu[b + 1]], sel[b], k[sl], v[sl], 0.4)
        np.testing.assert_array_equal(out[cu[b]:cu[b + 1]], ob)
        np.testing.assert_array_equal(lse[cu[b]:cu[b + 1]], lb)


# -------------------------------------------------------------------- end-to-end invariants

def _pipeline(lay, w, k):
    """deviation -> select -> scatter -> attention of the selected rows, all in the oracle."""
    _, dev_v, score = oracle.deviation(lay["v_fresh"], lay["v_cache"], reused=lay["reused"])
    n = w.n_ctx
    idx = oracle.select_topk(score, [0, n], [k])
    kc, vc = oracle._as_np(lay["k_cache"]).copy(), oracle._as_np(lay["v_cache"]).copy()
    li = torch.from_numpy(idx.astype(np.int64))
    oracle.scatter_kv(lay["k_fresh"][li], lay["v_fresh"][li], idx, kc, vc)
    return idx, kc, vc


def test_select_all_equals_full_prefill_and_none_equals_pure_reuse():
    w = synth.scaled(synth.TINY, 160, n_spans=3, span_lo=16, span_hi=40)
    lay = synth.make_layer(w)
    n_r = int(lay["reused"].sum())
    assert 0 < n_r < w.n_ctx
    # 100 %: every reused token recomputed -> the blended cache IS the fresh K/V, bit for bit
    idx, kc, vc = _pipeline(lay, w, n_r)
    np.testing.assert_array_equal(idx, np.nonzero(lay["reused"].numpy())[0])
    np.testing.assert_array_equal(kc, lay["k_fresh"].numpy())
    np.testing.assert_array_equal(vc, lay["v_fresh"].numpy())
    allpos = np.arange(w.n_ctx, dtype=np.int32)
    out_blend, _ = oracle.partial_attention(lay["q"], allpos, kc, vc, 1.0)
    np.testing.assert_allclose(out_blend, _sdpa_causal(lay["q"], lay["k_fresh"], lay["v_fresh"], 1.0), rtol=1e-10, atol=1e-12)
    # 0 %: nothing recomputed -> attention over the cache as reused
    idx0, kc0, vc0 = _pipeline(lay, w, 0)
    assert len(idx0) == 0
    out_reuse, _ = oracle.partial_attention(lay["q"], allpos, kc0, vc0, 1.0)
    np.testing.assert_allclose(out_reuse, _sdpa_causal(lay["q"], lay["k_cache"], lay["v_cache"], 1.0), rtol=1e-10, atol=1e-12)
    assert np.abs(out_reuse - out_blend).max() > 1e-3


def test_partial_rows_match_brute_force_full_recompute_for_every_k():
    # tiny: for every budget k, the selected rows' outputs equal the dense recompute over the
    # blended cache, and the error of the remaining rows shrinks to zero at k = n_R
    w = synth.scaled(synth.TINY, 48, n_spans=2, span_lo=8, span_hi=14)
    lay = synth.make_layer(w)
    n_r = int(lay["reused"].sum())
    for k in range(0, n_r + 1, 3):
        idx, kc, vc = _pipeline(lay, w, k)
        dense = _sdpa_causal(lay["q"], torch.from_numpy(kc), torch.from_numpy(vc), 1.0)
        out, _ = oracle.partial_attention(lay["q"][idx.astype(np.int64)], idx, kc, vc, 1.0)
        np.testing.assert_allclose(out, dense[idx], rtol=1e-10, atol=1e-12)


def test_value_jacobian_is_attention_matrix():
    # Sec. 4.1: dH/dV = A.  With Delta K = 0 the output is linear in V, so perturbing one value
    # entry of token i by delta changes row j by A[j,i]*delta and the column sum of the change
    # is alpha_i * delta: ties the attention oracle to the alpha oracle.
    n, hq, hk, d = 40, 2, 1, 4
    q, k, v = _rand((n, hq, d), torch.float32, 40), _rand((n, hk, d), torch.float32, 41), _rand((n, hk, d), torch.float32, 42)
    pos = np.arange(n, dtype=np.int32)
    h0, _ = oracle.partial_attention(q, pos, k, v, 0.5)
    v2 = v.clone()
    i, c, delta = 13, 2, 0.5
    v2[i, 0, c] += delta
    h1, _ = oracle.partial_attention(q, pos, k, v2, 0.5)
    ah, _ = oracle.alpha_prefill(q, k, 0.5)
    diff = h1 - h0
    np.testing.assert_allclose(diff[:, :, c].sum(0), ah[:, i] * delta, rtol=1e-9)
    assert np.abs(np.delete(diff, c, axis=2)).max() < 1e-14 and np.abs(diff[:i]).max() == 0


# ------------------------------------------------------------------------------- O7 decode

def test_decode_check_against_library_softmax():
    hq, hk, d = 6, 2, 16
    lens, pad = [57, 80, 5], 2
    off = np.cumsum([0] + [l + pad for l in lens])[:-1]
    rows = sum(lens) + pad * len(lens)
    k, v = _rand((rows, hk, d), torch.bfloat16, 50), _rand((rows, hk, d), torch.bfloat16, 51)
    q = _rand((3, hq, d), torch.bfloat16, 52, 0.5)
    g = torch.Generator().manual_seed(53)
    dev = torch.rand((hk, rows), generator=g)
    reused = (torch.rand(rows, generator=g) < 0.7).to(torch.uint8)
    kreq = [5, 9, 0]
    scale = 0.8
    idx, score, attn = oracle.decode_check(q, k, dev, reused, scale, off, lens, kreq, v_cache=v, want_attn=True)
    pos = 0
    for b in range(3):
        sl = slice(int(off[b]), int(off[b]) + lens[b])
        kk = k[sl].double().repeat_interleave(hq // hk, dim=1)             # [L, Hq, d]
        a = torch.softmax(torch.einsum("hd,ihd->hi", q[b].double(), kk) * scale, dim=-1)  # [Hq, L]
        mass = a.view(hk, hq // hk, -1).sum(1)                              # [Hkv, L]
        ref = (mass * dev[:, sl].double()).sum(0).numpy()
        m = reused[sl].numpy().astype(bool)
        np.testing.assert_allclose(score[sl][m], ref[m], rtol=1e-6)
        assert np.all(np.isneginf(score[sl][~m]))
        np.testing.assert_array_equal(idx[pos:pos + kreq[b]], _brute_select(score[sl], kreq[b]))
        pos += kreq[b]
        vv = v[sl].double().repeat_interleave(hq // hk, dim=1)
        np.testing.assert_allclose(attn[b], torch.einsum("hi,ihd->hd", a, vv).numpy(), rtol=1e-10)
    assert np.all(np.isnan(score[int(off[0]) + lens[0]: int(off[1])]))      # slack rows untouched


def test_decode_check_invariants_and_no_reselection():
    hq, hk, d, L = 4, 1, 8, 64
    k = _rand((L, hk, d), torch.float32, 54)
    q = _rand((1, hq, d), torch.float32, 55)
    dev = np.ones((hk, L), np.float32)
    reused = np.ones(L, np.uint8)
    idx, score, _ = oracle.decode_check(q, k, dev, reused, 0.3, [0], [L], [4])
    # dev == 1 and a single kv head: scores are the summed attention rows, total mass = Hq
    assert score.sum() == pytest.approx(hq, rel=1e-6)
    # after the write-back cleared the selected tokens they are never chosen again
    kc, vc = k.numpy().copy(), k.numpy().copy()
    oracle.scatter_kv(k[idx.astype(np.int64)], k[idx.astype(np.int64)], idx, kc, vc, reused, dev)
    idx2, score2, _ = oracle.decode_check(q, kc, dev, reused, 0.3, [0], [L], [4])
    assert not set(idx.tolist()) & set(idx2.tolist())
    assert np.all(np.isneginf(score2[idx]))
    # the decode row is the last row of the prefill attention: B=1 reduces to alpha's last row
    qfull = _rand((L, hq, d), torch.float32, 56)
    qfull[-1] = q[0]
    probs = _dense_causal_probs(qfull, k, 0.3)[:, -1, :].sum(0).numpy()
    _, score3, _ = oracle.decode_check(q, k, np.ones((hk, L), np.float32), np.ones(L, np.uint8), 0.3, [0], [L], [0])
    np.testing.assert_allclose(score3, probs, rtol=1e-6)


# ------------------------------------------------------------------------------- synth sanity

def test_synth_recipe_shapes_and_structure():
    lay = synth.make_layer(synth.TINY)
    r = lay["reused"].numpy()
    starts = np.nonzero(np.diff(np.concatenate([[0], r])) == 1)[0]
    ends = np.nonzero(np.diff(np.concatenate([r, [0]])) == -1)[0]
    assert len(starts) == 4 and np.all((ends - starts + 1 >= 32) & (ends - starts + 1 <= 128))
    assert torch.equal(lay["k_cache"][~lay["reused"].bool()], lay["k_fresh"][~lay["reused"].bool()])
    w = synth.scaled(synth.LLAMA, 8192)
    r = synth.make_spans(w, 1)
    assert 0.75 < r.mean() < 0.98
    lay2 = synth.make_layer(synth.TINY)
    assert all(torch.equal(lay[k], lay2[k]) for k in lay)          # seeded: same bits every time
    assert synth.recompute_budget(1000, 0.15) == 150 and synth.recompute_budget(1001, 0.1) == 101
