"""Parity at the benchmark's full sizes, in the launch configurations bench.py times: the
Llama-3.1-8B-shaped 32k layer, the Yi-1.5-9B-shaped 131k layer and the 64-request decode batch.
The oracle cannot recompute these outputs whole in reasonable time, so streaming steps (deviation,
select, scatter) are compared in full and attention / decode scores on sampled rows that the oracle
computes one by one, plus properties that hold at any size."""
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
CASE = [""]


def say(msg):
    CASE[0] = msg
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def attn_close(got, ref, mag, what=""):
    """The bf16 bar of attn_check.py: flat 2e-2 where the attended magnitude is at most 4,
    2e-2 + 2^-8 of it above; the slack each case used is logged."""
    check_attention(got, ref, mag, "bf16", f"{CASE[0]} {what}".strip())


def one_token_per_row_tile(n_sel, grp, tile_rows):
    """Indices into the selected-token list such that every row tile of the attention launch has
    at least one of its rows checked.  Rows are the flattened (selected token, head-in-group)
    pairs of a KV head, cut every tile_rows rows with the tiles aligned to the END of the list
    (the partly filled tile is the first); the row taken inside a tile moves from tile to tile so
    that over the launch every wave and lane position of a tile is visited.  The first two and
    the last two tokens are always included."""
    n_rows = n_sel * grp
    n_tiles = (n_rows + tile_rows - 1) // tile_rows
    picks = {0, min(1, n_sel - 1), max(n_sel - 2, 0), n_sel - 1}
    for t in range(n_tiles):
        hi = n_rows - (n_tiles - 1 - t) * tile_rows
        lo = max(hi - tile_rows, 0)
        picks.add((lo + (37 * t + 11) % (hi - lo)) // grp)
    return np.array(sorted(picks), dtype=np.int64)


def abs_bf16(a):
    """|x| on raw bf16 bit patterns (clear the sign bit)."""
    return (np.asarray(a).view(np.uint16) & np.uint16(0x7FFF)).view(np.uint16)


def prefill_layer(w, ratio, tile_rows, projected):
    """deviation -> select -> scatter -> attention at full size; returns nothing, asserts parity."""
    sh = B.shape_of(w)
    n, hk, hq, d = w.n_ctx, w.n_kv_heads, w.n_q_heads, w.head_dim
    lay = synth.make_layer(w, device=DEV, projected=projected)
    host = {k: v.cpu() for k, v in lay.items() if k != "q"}
    # a1, full comparison
    _, dev_ref, sc_ref = oracle.deviation(host["v_fresh"], host["v_cache"], reused=host["reused"])
    dev_v = torch.empty((hk, n), device=DEV)
    score = torch.empty((n,), device=DEV)
    B.kvs_deviation(sh, n, None, lay["v_fresh"], None, lay["v_cache"], lay["reused"], None, B.SCORE_V, None, dev_v, score)
    np.testing.assert_allclose(dev_v.cpu().numpy(), dev_ref, rtol=1e-5)
    fin = np.isfinite(sc_ref)
    sc = score.cpu().numpy()
    assert np.array_equal(np.isfinite(sc), fin)
    np.testing.assert_allclose(sc[fin], sc_ref[fin], rtol=1e-5)
    # a2 on the oracle's scores, bit-exact
    k = synth.recompute_budget(int(host["reused"].sum()), ratio)
    idx_ref = oracle.select_topk(sc_ref, [0, n], [k])
    idx = torch.empty((k,), dtype=torch.int32, device=DEV)
    B.kvs_select_topk(torch.from_numpy(sc_ref).to(DEV), [0, n], [k], idx)
    np.testing.assert_array_equal(idx.cpu().numpy(), idx_ref)
    # a4, full comparison
    li = torch.from_numpy(idx_ref.astype(np.int64))
    kc, vc = oracle._as_np(host["k_cache"]).copy(), oracle._as_np(host["v_cache"]).copy()
    reused = host["reused"].numpy().copy()
    oracle.scatter_kv(host["k_fresh"][li], host["v_fresh"][li], idx_ref, kc, vc, reused, dev_ref)
    gk, gv, gr = lay["k_cache"].clone(), lay["v_cache"].clone(), lay["reused"].clone()
    B.kvs_scatter_kv(sh, n, lay["k_fresh"][li.to(DEV)].contiguous(), lay["v_fresh"][li.to(DEV)].contiguous(), idx, k,
                     gk, gv, gr, dev_v)
    np.testing.assert_array_equal(oracle._as_np(gk.cpu()), kc)
    np.testing.assert_array_equal(oracle._as_np(gv.cpu()), vc)
    np.testing.assert_array_equal(gr.cpu().numpy(), reused)
    np.testing.assert_array_equal(dev_v.cpu().numpy() == 0, dev_ref == 0)
    # a3 with ALL selected queries in one launch (the timed configuration); sampled rows vs oracle
    q_sel = lay["q"][li.to(DEV)].contiguous()
    out = torch.empty((k, hq, d), dtype=torch.bfloat16, device=DEV)
    lse = torch.empty((k, hq), device=DEV)
    B.kvs_partial_attention(sh, [0], [n], [0, k], q_sel, idx, gk, gv, 1.0, out, lse)
    torch.cuda.synchronize()
    # at least one row of every row tile (x all heads: every KV head's tiles) against the oracle
    pick = one_token_per_row_tile(k, hq // hk, tile_rows)
    say(f"{CASE[0].split(';')[0]}; oracle on {len(pick)} of {k} selected tokens (one per {tile_rows}-row tile)")
    ref, ref_lse = oracle.partial_attention(q_sel[pick].cpu(), idx_ref[pick], kc, vc, 1.0)
    mag, _ = oracle.partial_attention(q_sel[pick].cpu(), idx_ref[pick], kc, abs_bf16(vc), 1.0)
    attn_close(out[pick].float().cpu().numpy(), ref, mag, "whole key ranges")
    np.testing.assert_allclose(lse[pick].cpu().numpy(), ref_lse, atol=2e-3)
    # properties over every row: finite, and |o| bounded by the largest |V| a row can see
    o = out.float()
    assert bool(torch.isfinite(o).all()) and bool(torch.isfinite(lse).all())
    assert float(o.abs().max()) <= float(gv.float().abs().max()) * (1 + 2.0 ** -7)
    # the same launch with a workspace, as bench.py passes one: small launches (the 5 % selection)
    # and contexts beyond the last-level cache (131k) then cut their key ranges into pieces
    ws = torch.empty(B.kvs_workspace_size("partial_attention", sh, 1, n, k), dtype=torch.uint8, device=DEV)
    out2 = torch.full_like(out, float("nan"))
    lse2 = torch.full_like(lse, float("nan"))
    B.kvs_partial_attention(sh, [0], [n], [0, k], q_sel, idx, gk, gv, 1.0, out2, lse2, workspace=ws)
    torch.cuda.synchronize()
    attn_close(out2[pick].float().cpu().numpy(), ref, mag, "with workspace")
    np.testing.assert_allclose(lse2[pick].cpu().numpy(), ref_lse, atol=2e-3)
    assert bool(torch.isfinite(out2.float()).all()) and bool(torch.isfinite(lse2).all())
    np.testing.assert_allclose(lse2.cpu().numpy(), lse.cpu().numpy(), atol=2e-3)
    del ws, out2, lse2
    return lay, gk, gv, gr, dev_v, idx_ref


# 5 %: few row tiles, the key range is cut into pieces; 15 % and 20 %: 72 and 96 row tiles per KV head on
# 32 compute units, every unit works through a planned share of them; 30 %: one workgroup per tile
@pytest.mark.parametrize("ratio", [0.05, 0.15, 0.20, 0.30])
def test_llama_32k_layer_full_size(ratio):
    say(f"llama 32k full size ratio {ratio}")
    # 128-row sampling also covers every tile of the 128-row kernel should the dispatch pick it
    prefill_layer(synth.LLAMA, ratio, tile_rows=128, projected=True)


@pytest.mark.timeout(900)
def test_qwen_8192_layer_full_size_with_exact_alpha():
    """The Qwen2.5-7B-shaped layer at its full 8192 tokens (28 query heads on 4 KV heads: groups of
    7, which do not divide a row tile): the magnitude-only path in full, then the whole of Alg. 1
    with the exact attention column mass -- kvs_attn_colsum -> kvs_deviation -> kvs_select_topk --
    against the oracle's alpha, scores and index set at this size."""
    w = synth.QWEN
    say("qwen 8192 full size")
    lay, gk, gv, gr, dev_v, idx_ref = prefill_layer(w, w.ratios[0], tile_rows=128, projected=False)
    sh = B.shape_of(w)
    n, hk, hq, d = w.n_ctx, w.n_kv_heads, w.n_q_heads, w.head_dim
    say("qwen 8192: exact alpha on the oracle side (a few 1e11 fp64 flop)")
    _, alpha_ref = oracle.alpha_prefill(lay["q"].cpu(), lay["k_fresh"].cpu(), 1.0)
    alpha = torch.empty((hk, n), device=DEV)
    ws = torch.empty(B.kvs_workspace_size("attn_colsum", sh, 1, n), dtype=torch.uint8, device=DEV)
    B.kvs_attn_colsum(sh, n, lay["q"], lay["k_fresh"], 1.0, alpha, ws)
    np.testing.assert_allclose(alpha.double().cpu().numpy(), alpha_ref, rtol=1e-4, atol=1e-7)
    np.testing.assert_allclose(alpha.double().sum(dim=1).cpu().numpy(), np.full(hk, float(n * (hq // hk))), rtol=1e-5)
    # scores with the device's alpha against the oracle's scores with its own alpha
    host = {k: lay[k].cpu() for k in ("v_fresh", "v_cache", "reused")}
    _, _, sc_ref = oracle.deviation(host["v_fresh"], host["v_cache"], reused=host["reused"], alpha=alpha_ref.astype(np.float32))
    score = torch.empty((n,), device=DEV)
    B.kvs_deviation(sh, n, None, lay["v_fresh"], None, lay["v_cache"], lay["reused"], alpha, B.SCORE_V, None, None, score)
    sc = score.cpu().numpy()
    fin = np.isfinite(sc_ref)
    assert np.array_equal(np.isfinite(sc), fin)
    np.testing.assert_allclose(sc[fin], sc_ref[fin], rtol=2e-4)      # alpha agrees to 1e-4, the deviation to 1e-5
    k = synth.recompute_budget(int(host["reused"].sum()), w.ratios[0])
    idx = torch.empty((k,), dtype=torch.int32, device=DEV)
    B.kvs_select_topk(score, [0, n], [k], idx)
    check_topk_band(idx.cpu().numpy(), sc_ref, k, rtol=4e-4)
    np.testing.assert_array_equal(idx.cpu().numpy(), oracle.select_topk(sc, [0, n], [k]))   # exact on its own scores
    # identical fp32 scores on both sides: bit-exact sets
    idx2 = torch.empty((k,), dtype=torch.int32, device=DEV)
    B.kvs_select_topk(torch.from_numpy(sc_ref).to(DEV), [0, n], [k], idx2)
    np.testing.assert_array_equal(idx2.cpu().numpy(), oracle.select_topk(sc_ref, [0, n], [k]))
    # the alpha-weighted ranking differs from the magnitude-only one (otherwise this test says nothing about alpha)
    assert len(set(idx2.cpu().numpy().tolist()) ^ set(idx_ref.tolist())) > 0


def test_yi_131k_layer_full_size():
    say("yi 131k full size")
    # one token per 256-row tile: each carries every key piece below its position through the merge
    prefill_layer(synth.YI, 0.10, tile_rows=256, projected=False)


def test_yi_131k_select_per_head_rows():
    """Top-k over 131k scores per KV head (four rows of one launch), bit-exact."""
    w = synth.YI
    say("yi 131k per-head top-k")
    lay = synth.make_layer(w, with_q=False, device=DEV)
    host_vf, host_vc = lay["v_fresh"].cpu(), lay["v_cache"].cpu()
    _, dev_ref, _ = oracle.deviation(host_vf, host_vc)
    n, hk = w.n_ctx, w.n_kv_heads
    rows = np.where(lay["reused"].cpu().numpy()[None, :] != 0, dev_ref, -np.inf).astype(np.float32)
    k = 12452
    ref = oracle.select_topk(rows.reshape(-1), [i * n for i in range(hk + 1)], [k] * hk)
    idx = torch.empty((hk * k,), dtype=torch.int32, device=DEV)
    scores = torch.from_numpy(rows.reshape(-1)).to(DEV)
    B.kvs_select_topk(scores, [i * n for i in range(hk + 1)], [k] * hk, idx)
    np.testing.assert_array_equal(idx.cpu().numpy(), ref)
    # with a workspace each row is cut into four parts that run on workgroups of their own
    ws = torch.empty(B.kvs_workspace_size("select_topk", B.shape_of(w), hk, hk * n), dtype=torch.uint8, device=DEV)
    idx.fill_(-1)
    B.kvs_select_topk(scores, [i * n for i in range(hk + 1)], [k] * hk, idx, ws)
    np.testing.assert_array_equal(idx.cpu().numpy(), ref)


def test_decode_batch_full_size():
    """64 requests with 4k-16k reused tokens each, one decode step: scores on sampled requests in
    full, top-k validity on every request, then write-back and the recompute attention sampled."""
    w = synth.DECODE
    say("decode batch 64 x (4k..16k)")
    sh = B.shape_of(w)
    batch = 64
    bt = synth.make_decode_batch(w, batch, 4096, 16384, 1, device=DEV)
    rows = bt["k_cache"].shape[0]
    off, lens = bt["ctx_off"], bt["ctx_len"].copy()
    hk, hq, d = w.n_kv_heads, w.n_q_heads, w.head_dim
    dev_v = torch.empty((hk, rows), device=DEV)
    B.kvs_deviation(sh, rows, None, bt["v_fresh"], None, bt["v_cache"], bt["reused"], None, B.SCORE_V, None, dev_v, None)
    gk, gv, gr = bt["k_cache"], bt["v_cache"], bt["reused"]
    for b in range(batch):                       # append the new token of each request
        r = int(off[b] + lens[b])
        gk[r] = bt["k_new"][0, b]
        gv[r] = bt["v_new"][0, b]
    lens = lens + 1
    kreq = [int(math.ceil(0.02 * l)) for l in lens]
    ws = torch.empty(B.kvs_workspace_size("decode_check", sh, batch, rows), dtype=torch.uint8, device=DEV)
    idx = torch.full((sum(kreq),), -1, dtype=torch.int32, device=DEV)
    score = torch.full((rows,), float("nan"), device=DEV)
    attn = torch.empty((batch, hq, d), dtype=torch.bfloat16, device=DEV)
    q_new = bt["q_new"][0].contiguous()
    B.kvs_decode_check(sh, rows, off, lens, q_new, gk, gv, dev_v, gr, 1.0, kreq, idx, score, attn, ws)
    torch.cuda.synchronize()
    sc, ix = score.cpu().numpy(), idx.cpu().numpy()
    # every request: ascending unique in-range candidates, and none better left out (on the GPU's own scores)
    cu = np.concatenate([[0], np.cumsum(kreq)])
    reused_h = gr.cpu().numpy()
    for b in range(batch):
        sl = slice(int(off[b]), int(off[b] + lens[b]))
        got = ix[cu[b]:cu[b + 1]]
        assert np.all(np.diff(got) > 0) and got[0] >= 0 and got[-1] < lens[b]
        assert np.all(reused_h[sl][got] == 1)
        row = sc[sl]
        chosen = np.zeros(lens[b], bool)
        chosen[got] = True
        assert row[chosen].min() >= row[~chosen].max()
    # sampled requests against the oracle (host copies of just those contexts)
    dev_h = dev_v.cpu().numpy()
    for b in (0, 17, 63):
        sl = slice(int(off[b]), int(off[b] + lens[b]))
        kc, vc = oracle._as_np(gk[sl].cpu()), oracle._as_np(gv[sl].cpu())
        ref_idx, ref_sc, ref_attn = oracle.decode_check(q_new[b:b + 1].cpu(), kc, dev_h[:, sl].copy(), reused_h[sl].copy(), 1.0,
                                                        [0], [lens[b]], [kreq[b]], v_cache=vc, want_attn=True)
        fin = np.isfinite(ref_sc)
        assert np.array_equal(np.isfinite(sc[sl]), fin)
        np.testing.assert_allclose(sc[sl][fin], ref_sc[fin], rtol=1e-5)
        _, _, mag_attn = oracle.decode_check(q_new[b:b + 1].cpu(), kc, dev_h[:, sl].copy(), reused_h[sl].copy(), 1.0,
                                             [0], [lens[b]], [0], v_cache=abs_bf16(vc), want_attn=True)
        attn_close(attn[b:b + 1].float().cpu().numpy(), ref_attn, mag_attn, f"decode attention output, request {b}")
        check_topk_band(ix[cu[b]:cu[b + 1]], ref_sc, kreq[b])
    # write-back + ragged recompute attention (the decode-stage a4 + a3), sampled against the oracle
    glob = torch.cat([idx[cu[b]:cu[b + 1]] + int(off[b]) for b in range(batch)]).contiguous()
    gl = glob.long()
    B.kvs_scatter_kv(sh, rows, bt["k_fresh"][gl].contiguous(), bt["v_fresh"][gl].contiguous(), glob, len(glob), gk, gv, gr, dev_v)
    assert int(gr[gl].sum()) == 0 and float(dev_v[:, gl].abs().max()) == 0.0
    g = torch.Generator(device=DEV).manual_seed(5)
    q_sel = (torch.randn((len(glob), hq, d), generator=g, device=DEV) / math.sqrt(d)).to(torch.bfloat16)
    out = torch.empty((len(glob), hq, d), dtype=torch.bfloat16, device=DEV)
    B.kvs_partial_attention(sh, off, lens, cu, q_sel, idx, gk, gv, 1.0, out)
    torch.cuda.synchronize()
    for b in (0, 17, 63):
        sl = slice(int(off[b]), int(off[b] + lens[b]))
        rows_b = np.arange(cu[b], cu[b + 1])[:: max(1, kreq[b] // 6)]
        kh, vh = oracle._as_np(gk[sl].cpu()), oracle._as_np(gv[sl].cpu())
        ref, _ = oracle.partial_attention(q_sel[rows_b].cpu(), ix[rows_b], kh, vh, 1.0)
        mag, _ = oracle.partial_attention(q_sel[rows_b].cpu(), ix[rows_b], kh, abs_bf16(vh), 1.0)
        attn_close(out[rows_b].float().cpu().numpy(), ref, mag, f"decode recompute, request {b}")


def test_attn_colsum_llama_32k_full_size():
    """The prefill column mass at 32k: the oracle needs every row's log-sum-exp for one column, so
    the comparison takes the last columns (column i needs the rows j >= i only) and the first
    column of a truncated context (alpha over the first m tokens is a problem of its own), plus
    what holds at any size: every softmax row sums to 1, the last column is at most one unit per
    head and the first at least one."""
    w = synth.LLAMA
    say("attention column mass, llama 32k")
    sh = B.shape_of(w)
    n, hk, hq, d = w.n_ctx, w.n_kv_heads, w.n_q_heads, w.head_dim
    grp = hq // hk
    lay = synth.make_layer(w, device=DEV)
    alpha = torch.empty((hk, n), device=DEV)
    ws = torch.empty(B.kvs_workspace_size("attn_colsum", sh, 1, n), dtype=torch.uint8, device=DEV)
    B.kvs_attn_colsum(sh, n, lay["q"], lay["k_fresh"], 1.0, alpha, ws)
    torch.cuda.synchronize()
    a = alpha.double().cpu().numpy()
    assert np.all(np.isfinite(a)) and np.all(a > 0)
    np.testing.assert_allclose(a.sum(axis=1), np.full(hk, float(n * grp)), rtol=1e-5)
    assert np.all(a[:, -1] <= grp) and np.all(a[:, 0] >= grp)
    # last m columns against the oracle's rows
    m = 8
    q_tail, k_all = lay["q"][n - m:].cpu(), lay["k_fresh"].cpu()
    _, lse = oracle.partial_attention(q_tail, np.arange(n - m, n, dtype=np.int32), k_all, lay["v_fresh"].cpu(), 1.0)
    qf, kf = q_tail.double().numpy(), k_all[n - m:].double().numpy()
    ref = np.zeros((hk, m))
    for j in range(m):
        for h in range(hq):
            s = kf[: j + 1, h // grp] @ qf[j, h]
            ref[h // grp, : j + 1] += np.exp(s - lse[j, h])
    np.testing.assert_allclose(a[:, n - m:], ref, rtol=1e-4, atol=1e-7)
    # the same kernel on the first 1500 tokens, in full against the oracle
    m2 = 1500
    _, ref2 = oracle.alpha_prefill(lay["q"][:m2].cpu(), k_all[:m2], 1.0)
    alpha2 = torch.empty((hk, m2), device=DEV)
    B.kvs_attn_colsum(sh, m2, lay["q"], lay["k_fresh"], 1.0, alpha2, ws)
    np.testing.assert_allclose(alpha2.double().cpu().numpy(), ref2, rtol=1e-4, atol=1e-7)
