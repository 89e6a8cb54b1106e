"""The decode stage as the paper runs it (Sec. 4.2; App. A: the candidates are the tokens that were
reused during prefill and have not been recomputed since): many steps in a row, each appending one
token per request, re-scoring the remaining reused entries against the new token's attention,
recomputing the best 2 % and writing them back, until the pool of candidates is empty and the
check degenerates to k = 0.

Every step runs kvs_decode_check -> kvs_scatter_kv -> kvs_partial_attention on the device, the
index list going from one call to the next without a host copy in between; the host only clips
k_req to the candidates each request has left (it knows the count: what it started with minus
what it asked for so far).  The oracle runs the same loop on its own state; the two sides rank
their own scores, which agree to 1e-5, so a step's index set is first checked for validity
against the oracle's scores (everything clearly above the k-th score in, everything clearly below
out) and the oracle's state then follows the device's choice, which keeps the two states
comparable bit for bit after every step.
"""
import math
import sys

import numpy as np
import pytest
import torch

import oracle
from attn_check import check_attention, check_topk_band
from paper_2503_16525_amd import binding as B
from paper_2503_16525_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def abs_bf16(a):
    return np.asarray(a).view(np.uint16) & np.uint16(0x7FFF)


def run_decode_loop(batch, len_lo, len_hi, steps, attn_every, half_reused_request=None):
    w = synth.DECODE
    sh = B.shape_of(w)
    hk, hq, d = w.n_kv_heads, w.n_q_heads, w.head_dim
    bt = synth.make_decode_batch(w, batch, len_lo, len_hi, steps, salt=9)
    rows = bt["k_cache"].shape[0]
    off, lens0 = bt["ctx_off"], bt["ctx_len"].copy()
    reused0 = bt["reused"].numpy().copy()
    if half_reused_request is not None:     # one request whose pool is half the size: it drains early
        b = half_reused_request
        reused0[off[b] + lens0[b] // 2: off[b] + lens0[b]] = 0
    # "prefill": the stored deviation, each side on its own path
    _, dev_ref, _ = oracle.deviation(bt["v_fresh"], bt["v_cache"], reused=reused0)
    g = {k: (v.to(DEV) if isinstance(v, torch.Tensor) else v) for k, v in bt.items()}
    gr = torch.from_numpy(reused0).to(DEV)
    dev_gpu = torch.empty((hk, rows), device=DEV)
    B.kvs_deviation(sh, rows, None, g["v_fresh"], None, g["v_cache"], gr, None, B.SCORE_V, None, dev_gpu, None)
    kc, vc = oracle._as_np(bt["k_cache"]).copy(), oracle._as_np(bt["v_cache"]).copy()
    reused = reused0.copy()
    gk, gv = g["k_cache"].clone(), g["v_cache"].clone()
    ws = torch.empty(B.kvs_workspace_size("decode_check", sh, batch, rows), dtype=torch.uint8, device=DEV)
    k_max = sum(int(math.ceil(0.02 * (l + steps))) for l in lens0)
    ws_att = torch.empty(B.kvs_workspace_size("partial_attention", sh, batch, rows, k_max), dtype=torch.uint8, device=DEV)
    remaining = np.array([int(reused0[off[b]: off[b] + lens0[b]].sum()) for b in range(batch)])
    ever = [set() for _ in range(batch)]
    lens = lens0.copy()
    gen = torch.Generator().manual_seed(77)
    first_idle = None
    n_attn_checked = 0
    for step in range(steps):
        for b in range(batch):                     # the new token's K/V, fresh: never a candidate
            r = int(off[b] + lens[b])
            kc[r] = oracle._as_np(bt["k_new"][step, b])
            vc[r] = oracle._as_np(bt["v_new"][step, b])
        rr = torch.from_numpy((off + lens).astype(np.int64)).to(DEV)
        gk[rr] = g["k_new"][step]
        gv[rr] = g["v_new"][step]
        lens = lens + 1
        want = np.array([int(math.ceil(0.02 * l)) for l in lens])
        kreq = np.minimum(want, remaining)          # the host-side clip to what is left
        n_sel = int(kreq.sum())
        cu = np.concatenate([[0], np.cumsum(kreq)]).astype(np.int64)
        say(f"decode loop step {step}: k_req {kreq.tolist()} of {remaining.tolist()} left")
        # ---- device: a5 -> a4 -> a3, indices stay on the device --------------------------------
        state_before = (gk.clone(), gv.clone(), gr.clone(), dev_gpu.clone()) if n_sel == 0 else None
        idx = torch.full((max(n_sel, 1),), -1, dtype=torch.int32, device=DEV)
        score = torch.full((rows,), float("nan"), device=DEV)
        q_step = g["q_new"][step].contiguous()
        B.kvs_decode_check(sh, rows, off, lens, q_step, gk, None, dev_gpu, gr, 1.0, kreq.tolist(), idx, score, None, ws)
        row_base = torch.from_numpy(np.repeat(off, kreq).astype(np.int32)).to(DEV)
        glob = (idx[:n_sel] + row_base).contiguous()
        gl = glob.long()
        q_sel = (torch.randn((max(n_sel, 1), hq, d), generator=gen) / math.sqrt(d)).to(torch.bfloat16)[:n_sel]
        q_sel_g = q_sel.to(DEV)
        out = torch.full((max(n_sel, 1), hq, d), float("nan"), dtype=torch.bfloat16, device=DEV)
        B.kvs_scatter_kv(sh, rows, g["k_fresh"][gl].contiguous(), g["v_fresh"][gl].contiguous(), glob, n_sel,
                         gk, gv, gr, dev_gpu)
        B.kvs_partial_attention(sh, off, lens, cu, q_sel_g, idx, gk, gv, 1.0, out, None, ws_att)
        torch.cuda.synchronize()
        ix = idx[:n_sel].cpu().numpy()
        # ---- oracle on its own state --------------------------------------------------------------
        ref_idx, ref_score, _ = oracle.decode_check(bt["q_new"][step], kc, dev_ref, reused, 1.0, off, lens, kreq.tolist())
        sc = score.cpu().numpy()
        for b in range(batch):
            sl = slice(int(off[b]), int(off[b] + lens[b]))
            inf = np.isneginf(ref_score[sl])
            assert np.array_equal(np.isneginf(sc[sl]), inf), f"step {step}, request {b}: candidate sets differ"
            np.testing.assert_allclose(sc[sl][~inf], ref_score[sl][~inf], rtol=1e-5, atol=0)
            got = ix[cu[b]:cu[b + 1]]
            check_topk_band(got, ref_score[sl], int(kreq[b]))
            assert np.all(reused[sl][got] == 1), "a token that is no longer a candidate was returned"
            assert not (ever[b] & set(got.tolist())), f"step {step}, request {b}: an index came back a second time"
            ever[b].update(got.tolist())
        same = np.array_equal(ix, ref_idx)
        # the oracle's state follows the device's (validated) choice
        glob_h = (ix + np.repeat(off, kreq)).astype(np.int32)
        li = torch.from_numpy(glob_h.astype(np.int64))
        oracle.scatter_kv(bt["k_fresh"][li], bt["v_fresh"][li], glob_h, kc, vc, reused, dev_ref)
        np.testing.assert_array_equal(gr.cpu().numpy(), reused)
        np.testing.assert_array_equal(dev_gpu.cpu().numpy() == 0, dev_ref == 0)
        if step % 8 == 0 or n_sel == 0:
            np.testing.assert_array_equal(oracle._as_np(gk.cpu()), kc)
            np.testing.assert_array_equal(oracle._as_np(gv.cpu()), vc)
        remaining = remaining - kreq
        if n_sel == 0:
            # nothing left to recompute: the three calls change nothing and write nothing
            if first_idle is None:
                first_idle = step
            for a, b_ in zip(state_before, (gk, gv, gr, dev_gpu)):
                assert torch.equal(a, b_)
            assert int(idx[0]) == -1 and bool(torch.isnan(out.float()).all())
            continue
        if step % attn_every == 0 or ((remaining == 0) & (kreq > 0)).any():    # also whenever a pool just emptied
            ref, _ = oracle.partial_attention(q_sel, ix, kc, vc, 1.0, off, lens, cu)
            mag, _ = oracle.partial_attention(q_sel, ix, kc, abs_bf16(vc), 1.0, off, lens, cu)
            check_attention(out[:n_sel].float().cpu().numpy(), ref, mag, "bf16",
                            f"decode loop step {step} ({n_sel} recomputed tokens, indices {'equal to' if same else 'a valid variant of'} the oracle's)")
            n_attn_checked += 1
    assert int(remaining.sum()) == 0, "the pool did not drain"
    assert first_idle is not None and first_idle < steps - 1, "no k = 0 step was reached"
    was_candidate = torch.from_numpy(reused0.astype(bool)).to(DEV)
    assert int(gr.sum()) == 0 and float(dev_gpu[:, was_candidate].abs().max()) == 0.0
    for b in range(batch):      # every reused token of the initial context was recomputed exactly once
        assert ever[b] == set(np.nonzero(reused0[off[b]: off[b] + lens0[b]])[0].tolist())
    assert n_attn_checked >= 3
    return first_idle


def test_decode_loop_until_the_pool_is_empty():
    """8 requests of 700-2000 reused tokens, 128 steps: the pools drain after ~50 steps (request 2
    after ~25: only half of its context is reused), the remaining steps are k = 0 no-ops."""
    first_idle = run_decode_loop(batch=8, len_lo=700, len_hi=2000, steps=128, attn_every=16, half_reused_request=2)
    assert 45 <= first_idle <= 55
