"""Seeded random cases on top of the hand-picked ones: the matcher, the three top-k entry points, partial
attention (with and without a workspace, ragged batches, every head layout the kernels special-case) and the
decode check, each against the oracle.  The generators draw sizes log-uniformly so that one-element, one-tile
and many-tile inputs all turn up; every case prints what it is before it runs."""
import math

import numpy as np
import pytest
import torch

import oracle
from attn_check import check_topk_band
from paper_2503_16525_amd import binding as B
from paper_2503_16525_amd import synth
import test_gpu_match as TM
import test_gpu_parity as TP

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("seed", range(12))
def test_random_match(seed):
    rng = np.random.default_rng(10_000 + seed)
    vocab = int(rng.choice([2, 3, 5, 17, 100, 5000, 128000]))
    w = int(rng.choice([1, 2, 3, 4, 7, 16, 31, 64, 200, 769, 1000]))
    m = int(rng.choice([1, 2, 13, 251, 65521, 4294967291]))
    b = int(rng.choice([1, 2, 31, 1000003, 4294967290]))
    nt, nc = int(rng.integers(0, 20000)), int(rng.integers(0, 20000))
    kind = int(rng.integers(0, 4))
    TM.say(f"random match seed={seed} vocab={vocab} w={w} m={m} b={b} n_target={nt} n_candidate={nc} kind={kind}")
    cand = rng.integers(0, vocab, size=nc)
    if kind == 0 or nc == 0:
        targ = rng.integers(0, vocab, size=nt)
    else:   # the target is pieces of the candidate (some periodic) with fresh tokens between them
        parts, tot = [], 0
        while tot < nt:
            if rng.random() < 0.7:
                length, start = int(rng.integers(1, 600)), int(rng.integers(0, max(nc - 1, 1)))
                p = cand[start:start + length]
                if kind == 3 and len(p) > 4:
                    p = np.tile(p[:4], len(p) // 4 + 1)[:len(p)]
            else:
                p = rng.integers(0, vocab, size=int(rng.integers(1, 100)))
            parts.append(p)
            tot += len(p)
        targ = np.concatenate(parts)[:nt] if parts else np.zeros(0, dtype=np.int64)
    TM.check(targ, cand, w, b, m)


@pytest.mark.parametrize("seed", range(24))
def test_random_select(seed):
    rng = np.random.default_rng(20_000 + seed)
    rows = int(rng.choice([1, 1, 1, 2, 5, 17]))
    lens = [int(rng.choice([1, 7, 64, 1000, 4097, 20000, 49152, 49153, 70000, 150000])) for _ in range(rows)]
    if rows > 1:
        lens = [min(n, 30000) for n in lens]
    n = sum(lens)
    kind = int(rng.integers(0, 5))
    if kind == 0:
        s = rng.lognormal(-3, 1.5, n)
    elif kind == 1:
        s = np.round(rng.lognormal(-3, 1.5, n), 2)                       # many ties
    elif kind == 2:
        s = rng.choice([0.0, -0.0, 1.0, -np.inf, 3.5, 1e-42, -2.0], size=n)
    elif kind == 3:
        s = rng.normal(size=n) * 10.0 ** rng.integers(-30, 30, size=n)
    else:
        s = np.full(n, 0.25)
    s = s.astype(np.float32)
    if kind != 2 and n > 10:
        s[rng.integers(0, n, size=n // 10)] = -np.inf
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    ks = [int(rng.choice([0, 1, n_r, n_r // 2, max(n_r // 50, 1), n_r - 1 if n_r > 1 else 1])) for n_r in lens]
    TP.say(f"random select seed={seed} rows={rows} lens={lens[:6]} k={ks[:6]} kind={kind}")
    ref = oracle.select_topk(s, off, ks)
    for ws in (False, True):
        np.testing.assert_array_equal(TP.gpu_select(s, off, ks, with_workspace=ws), ref)
    if max(lens) <= 262144 and rows <= 64:
        out = torch.full((max(sum(ks), 1),), -7, dtype=torch.int32, device=DEV)
        B.kvs_select_topk_static(torch.from_numpy(s).to(DEV), off, ks, out)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(out.cpu().numpy()[:sum(ks)], ref)


@pytest.mark.parametrize("seed", range(24))
def test_random_attention_batch(seed):
    rng = np.random.default_rng(50_000 + seed)
    hk, grp = [(8, 4), (4, 7), (4, 8), (2, 1), (1, 1), (8, 1), (16, 2), (2, 16)][seed % 8]
    w = synth.scaled(synth.LLAMA, 0, n_q_heads=hk * grp, n_kv_heads=hk)
    n_req = int(rng.choice([1, 1, 1, 2, 3, 5, 8]))
    hi = [300, 3000, 40000][int(rng.integers(0, 3))]
    lens = [int(math.exp(rng.uniform(0, math.log(hi)))) for _ in range(n_req)]
    lens = [max(1, min(n, 40000 // n_req + 1)) for n in lens]
    pad = int(rng.integers(0, 3))
    off = np.cumsum([0] + [n + pad for n in lens])[:-1]
    rows = sum(lens) + pad * n_req
    g = torch.Generator().manual_seed(60_000 + seed)
    k = (torch.randn((rows, hk, w.head_dim), generator=g) * float(rng.choice([1.0, 1.0, 3.0]))).to(torch.bfloat16)
    v = torch.randn((rows, hk, w.head_dim), generator=g).to(torch.bfloat16)
    sel = []
    for n in lens:
        cnt = int(rng.choice([0, 1, min(n, 7), min(n, 64), min(n, 65), min(n, int(rng.integers(1, 2500))), n if n < 3000 else 100]))
        kind = int(rng.integers(0, 5))
        if kind == 0:
            p = np.arange(n - cnt, n)
        elif kind == 1:
            p = np.arange(0, cnt)
        elif kind == 2:
            p = np.sort(rng.choice(n, size=cnt, replace=False))
        elif kind == 3:
            p = rng.permutation(rng.choice(n, size=cnt, replace=False))
        else:
            p = np.sort(rng.integers(0, n, size=cnt))                    # with repeats
        sel.append(p.astype(np.int32))
    cu = np.cumsum([0] + [len(x) for x in sel])
    ns = int(cu[-1])
    TP.say(f"random attention seed={seed} heads {hk}x{grp} contexts={lens} selected={[len(x) for x in sel]} pad={pad}")
    if ns == 0:
        return
    q = (torch.randn((ns, w.n_q_heads, w.head_dim), generator=g) / math.sqrt(w.head_dim)).to(torch.bfloat16)
    pos = np.concatenate(sel)
    got_ws, lse_ws = TP.run_gpu_attention(w, q, pos, k, v, 1.0, off, lens, cu)
    got_no, lse_no = TP.run_gpu_attention(w, q, pos, k, v, 1.0, off, lens, cu, with_workspace=False)
    assert np.all(np.isfinite(got_ws)) and np.all(np.isfinite(lse_ws)) and np.all(np.isfinite(got_no))
    np.testing.assert_allclose(lse_ws, lse_no, atol=2e-3)
    for b in range(n_req):
        if cu[b + 1] == cu[b]:
            continue
        pick = np.unique(np.concatenate([rng.integers(cu[b], cu[b + 1], size=10), [cu[b], cu[b + 1] - 1]]))
        ref, ref_lse = oracle.partial_attention(q[pick], pos[pick], k, v, 1.0, [off[b]], [lens[b]], [0, len(pick)])
        mag = TP.attn_magnitude(q[pick], pos[pick], k, v, 1.0, [off[b]], [lens[b]], [0, len(pick)])
        TP.assert_attn_close(got_ws[pick], ref, w, mag)
        TP.assert_attn_close(got_no[pick], ref, w, mag)
        np.testing.assert_allclose(lse_ws[pick], ref_lse, atol=2e-3)


@pytest.mark.parametrize("seed", range(16))
def test_random_decode_check(seed):
    rng = np.random.default_rng(70_000 + seed)
    dtype, d, hq, hk = [("bf16", 128, 32, 8), ("bf16", 128, 28, 4), ("bf16", 128, 32, 4), ("bf16", 128, 8, 8), ("bf16", 64, 24, 2),
                        ("f32", 64, 8, 4), ("f32", 128, 4, 4), ("bf16", 128, 64, 2)][seed % 8]
    w = synth.scaled(synth.DECODE, 0, dtype=dtype, head_dim=d, n_q_heads=hq, n_kv_heads=hk)
    batch = int(rng.choice([1, 1, 1, 2, 5, 17, 70]))
    hi = int(rng.choice([40, 700, 5000, 20000])) if batch > 1 else int(rng.choice([40, 700, 12288, 12289, 14000, 40000]))
    hi = max(2, min(hi, 60000 // batch))
    lo = hi if batch == 1 else int(rng.integers(1, hi))
    bt = synth.make_decode_batch(w, batch, lo, hi, 1, salt=int(rng.integers(0, 1 << 20)))
    rows = bt["k_cache"].shape[0]
    off, lens = bt["ctx_off"], bt["ctx_len"].copy() + 1
    sh = TP.shape_for(w)
    kreq = [int(rng.choice([0, 1, max(1, int(0.02 * n)), min(int(n) - 1, int(0.3 * n) + 1)])) for n in lens]
    TP.say(f"random decode check seed={seed} {dtype} d{d} {hq}/{hk} batch={batch} contexts={list(map(int, lens))[:6]} k={kreq[:6]}")
    _, dev_ref, _ = oracle.deviation(bt["v_fresh"], bt["v_cache"], reused=bt["reused"])
    g = TP.to_dev(bt)
    dev_gpu = torch.from_numpy(dev_ref).to(DEV)
    reused = bt["reused"].numpy().copy()
    reused[rng.random(rows) < 0.1] = 0                                   # rows recomputed earlier: no candidates
    gr = torch.from_numpy(reused).to(DEV)
    kreq = [min(kq, int(reused[int(off[b]):int(off[b] + lens[b])].sum())) for b, kq in enumerate(kreq)]
    kc = oracle._as_np(bt["k_cache"])
    ref_idx, ref_score, _ = oracle.decode_check(bt["q_new"][0], kc, dev_ref, reused, 1.0, off, lens, kreq)
    ws = torch.empty(B.kvs_workspace_size("decode_check", sh, batch, rows), dtype=torch.uint8, device=DEV)
    idx = torch.full((max(sum(kreq), 1),), -1, dtype=torch.int32, device=DEV)
    score = torch.full((rows,), float("nan"), device=DEV)
    B.kvs_decode_check(sh, rows, off, lens, g["q_new"][0].contiguous(), g["k_cache"], None, dev_gpu, gr, 1.0, kreq,
                       idx, score, None, ws)
    torch.cuda.synchronize()
    sc, ix = score.cpu().numpy(), idx.cpu().numpy()
    p = 0
    for b in range(batch):
        sl = slice(int(off[b]), int(off[b] + lens[b]))
        TP.assert_scores_close(sc[sl], ref_score[sl])
        check_topk_band(ix[p:p + kreq[b]], ref_score[sl], kreq[b])
        # and bit for bit the ranking of the call's own scores
        np.testing.assert_array_equal(ix[p:p + kreq[b]], oracle.select_topk(sc[sl], [0, int(lens[b])], [kreq[b]]))
        p += kreq[b]
