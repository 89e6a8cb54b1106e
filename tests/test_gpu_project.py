"""kvs_project_qkv (App. D.1: a later layer's Q/K/V of the tokens selected earlier) against the oracle.

Tolerance, from the arithmetic: the device multiplies bf16 inputs exactly, accumulates in fp32 (error below
hidden * 2^-24 * sum |x w|, under 1e-4 for unit-variance inputs at hidden 4096), rotates in fp32 and rounds
once to bf16 (half an ulp: 2^-9 relative).  Asserted: |got - ref| <= 2^-8 |ref| + 2e-4 on every element."""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2503_16525_amd import binding as B
from paper_2503_16525_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def run_gpu(w, x, wt, rows, pos, rope):
    sh = B.shape_of(w)
    n_sel = x.shape[0] if rows is None else len(rows)
    q = torch.full((n_sel, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.bfloat16, device=DEV)
    k = torch.full((n_sel, w.n_kv_heads, w.head_dim), float("nan"), dtype=torch.bfloat16, device=DEV)
    v = torch.full((n_sel, w.n_kv_heads, w.head_dim), float("nan"), dtype=torch.bfloat16, device=DEV)
    dev = lambda a, dt: None if a is None else torch.from_numpy(np.asarray(a, dtype=dt)).to(DEV)
    B.kvs_project_qkv(sh, x.to(DEV), dev(rows, np.int32), dev(pos, np.int32), n_sel, wt.to(DEV),
                      None if rope is None else torch.from_numpy(rope).to(DEV), q, k, v)
    torch.cuda.synchronize()
    return [t.float().cpu().numpy().astype(np.float64) for t in (q, k, v)]


def compare(got, ref, what):
    worst = 0.0
    for name, g, r in zip("qkv", got, ref):
        assert np.all(np.isfinite(g)), f"{what}: {name} has unwritten or non-finite entries"
        tol = 2.0 ** -8 * np.abs(r) + 2e-4
        err = np.abs(g - r)
        assert np.all(err <= tol), f"{what}: {name} max err {err.max():.3e}, worst ratio {(err / tol).max():.2f}"
        worst = max(worst, float((err / tol).max()))
    say(f"  {what}: worst error / tolerance {worst:.2f}")


CASES = [
    # name, q heads, kv heads, hidden, tokens, selected, gather, rotary
    ("g2-gather-rope", 4, 2, 256, 700, 300, True, True),
    ("qwen-heads-513", 28, 4, 512, 900, 513, True, True),
    ("dense-rows-no-rope", 8, 4, 128, 256, 256, False, False),
    ("one-token", 4, 2, 64, 50, 1, True, True),
    ("257-rope-no-gather", 6, 1, 192, 257, 257, False, True),
    ("llama-heads-hidden-1024", 32, 8, 1024, 2000, 640, True, True),
]


@pytest.mark.parametrize("name,hq,hk,hidden,n,n_sel,gather,rotary", CASES, ids=[c[0] for c in CASES])
def test_project_qkv_parity(name, hq, hk, hidden, n, n_sel, gather, rotary):
    say(f"project_qkv {name}")
    w = synth.scaled(synth.LLAMA, n, n_q_heads=hq, n_kv_heads=hk)
    x, wt = synth.make_projection(w, hidden)
    rng = np.random.default_rng(len(name))
    rows = np.sort(rng.choice(n, size=n_sel, replace=False)).astype(np.int32) if gather else None
    pos = rows if gather else np.arange(n_sel, dtype=np.int32)
    if name == "one-token":
        rows = pos = np.array([n - 1], dtype=np.int32)
    rope = synth.make_rope_table(n, w.head_dim) if rotary else None
    got = run_gpu(w, x, wt, rows, pos if rotary else None, rope)
    ref = oracle.project_qkv(x, wt, hq, hk, w.head_dim, rows=rows, pos=pos if rotary else None, rope=rope)
    compare(got, ref, name)


def test_project_qkv_rows_may_repeat_and_come_unsorted():
    say("project_qkv unsorted rows with repeats")
    w = synth.scaled(synth.LLAMA, 400, n_q_heads=4, n_kv_heads=2)
    x, wt = synth.make_projection(w, 128)
    rows = np.array([399, 0, 17, 17, 250, 3] * 50, dtype=np.int32)
    rope = synth.make_rope_table(400, w.head_dim)
    got = run_gpu(w, x, wt, rows, rows, rope)
    ref = oracle.project_qkv(x, wt, 4, 2, w.head_dim, rows=rows, pos=rows, rope=rope)
    compare(got, ref, "unsorted")


def test_project_qkv_llama_layer_full_size():
    """the 32k Llama-shaped layer at ratio 0.15: 4.6k selected tokens x 4096 -> 6144 features; the oracle follows
    every feature of three tokens from every 256-token tile (first, last and one in between)"""
    w = synth.LLAMA
    say("project_qkv llama 32k full size")
    x, wt = synth.make_projection(w, w.hidden)
    lay_reused = synth.make_spans(w, synth.layer_seed(w, 0))
    n_sel = synth.recompute_budget(int(lay_reused.sum()), 0.15)
    rng = np.random.default_rng(5)
    rows = np.sort(rng.choice(w.n_ctx, size=n_sel, replace=False)).astype(np.int32)
    rope = synth.make_rope_table(w.n_ctx, w.head_dim)
    got = run_gpu(w, x, wt, rows, rows, rope)
    picks = []
    for t0 in range(0, n_sel, 256):
        t1 = min(t0 + 256, n_sel)
        picks += [t0, t1 - 1, int(rng.integers(t0, t1))]
    picks = np.array(sorted(set(picks)))
    ref = oracle.project_qkv(x, wt, w.n_q_heads, w.n_kv_heads, w.head_dim, rows=rows[picks], pos=rows[picks], rope=rope)
    compare([g[picks] for g in got], ref, f"llama 32k, {picks.size} sampled tokens")
    # every output was written and is of the expected size (unit-variance features)
    for g in got:
        assert np.all(np.isfinite(g)) and 0.9 < g.std() < 1.1


def test_project_qkv_rejects_what_is_not_built():
    w = synth.scaled(synth.LLAMA, 64, n_q_heads=4, n_kv_heads=2)
    x, wt = synth.make_projection(w, 64)
    sh = B.shape_of(w)
    q = torch.empty((64, 4, 128), dtype=torch.bfloat16, device=DEV)
    k = torch.empty((64, 2, 128), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(B.KvsError):      # hidden not a multiple of 64
        B.kvs_project_qkv(sh, x[:, :48].contiguous().to(DEV), None, None, 64, wt[:, :48].contiguous().to(DEV), None, q, k, k.clone())
    with pytest.raises(B.KvsError):      # more tokens selected than x has rows, without a row list
        B.kvs_project_qkv(sh, x.to(DEV), None, None, 65, wt.to(DEV), None, q, k, k.clone())
    B.kvs_project_qkv(sh, x.to(DEV), None, None, 0, wt.to(DEV), None, q, k, k.clone())     # nothing selected: no-op
