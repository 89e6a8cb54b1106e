"""kvs_deviation_topk (Alg. 1 steps 3-4 in one call) against the two separate calls, bit for bit,
and against the oracle: scores to 1e-5, the index list exact on the scores the call itself
wrote.  The cases aim at what the fused path adds: the key histogram that the scoring kernel
fills and the selecting kernel clears (so every case here also checks that the call before it
left the histogram clean), thresholds inside large ties, more requested entries than finite
scores, rows at the edges of the register-resident range."""
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


def fused_and_separate(w, lay, k, alpha=None, mode=B.SCORE_V, with_score=True, reused="layer"):
    sh = B.shape_of(w)
    n, hk = w.n_ctx, w.n_kv_heads
    g = {key: v.to(DEV) for key, v in lay.items() if isinstance(v, torch.Tensor)}
    ru = g["reused"] if reused == "layer" else reused
    al = alpha.to(DEV) if alpha is not None else None
    kf, kc = (g["k_fresh"], g["k_cache"]) if mode == B.SCORE_KV else (None, None)
    dev_a, sc_a = torch.empty((hk, n), device=DEV), torch.empty((n,), device=DEV)
    idx_a = torch.full((k,), -1, dtype=torch.int32, device=DEV)
    B.kvs_deviation(sh, n, kf, g["v_fresh"], kc, g["v_cache"], ru, al, mode, None, dev_a, sc_a)
    B.kvs_select_topk(sc_a, [0, n], [k], idx_a)
    dev_b = torch.empty((hk, n), device=DEV)
    sc_b = torch.full((n,), float("nan"), device=DEV) if with_score else None
    idx_b = torch.full((k,), -2, dtype=torch.int32, device=DEV)
    ws = torch.empty(B.kvs_workspace_size("select_topk", sh, 1, n), dtype=torch.uint8, device=DEV)
    B.kvs_deviation_topk(sh, n, kf, g["v_fresh"], kc, g["v_cache"], ru, al, mode, None, dev_b, sc_b, k, idx_b, ws)
    torch.cuda.synchronize()
    assert torch.equal(dev_a, dev_b)
    if with_score:
        assert torch.equal(sc_a.view(torch.int32), sc_b.view(torch.int32))
    np.testing.assert_array_equal(idx_b.cpu().numpy(), idx_a.cpu().numpy())
    # and the list is the exact top-k of those scores by the oracle's definition
    np.testing.assert_array_equal(idx_b.cpu().numpy(), oracle.select_topk(sc_a.cpu().numpy(), [0, n], [k]))
    return sc_a.cpu().numpy(), idx_b.cpu().numpy()


CASES = [
    ("tiny-f32", synth.TINY, 0.15),
    ("llama-4133", synth.scaled(synth.LLAMA, 4133), 0.15),
    ("qwen-8192", synth.QWEN, 0.10),
    ("llama-32768", synth.LLAMA, 0.15),
    ("llama-1", synth.scaled(synth.LLAMA, 1, coverage=1.0), 1.0),
    ("llama-63", synth.scaled(synth.LLAMA, 63, span_mean=8.0), 0.5),
    ("llama-1023", synth.scaled(synth.LLAMA, 1023, span_mean=64.0), 0.3),
    ("llama-1025", synth.scaled(synth.LLAMA, 1025, span_mean=64.0), 0.3),
    ("llama-12288-two-calls", synth.scaled(synth.LLAMA, 12288), 0.3),
    ("llama-12289", synth.scaled(synth.LLAMA, 12289), 0.3),
    ("llama-49153", synth.scaled(synth.LLAMA, 49153), 0.3),
    ("yi-131072", synth.YI, 0.10),
    ("one-head-262144", synth.scaled(synth.LLAMA, 262144, n_kv_heads=1, n_q_heads=1, head_dim=64), 0.1),
    ("one-head-262145-two-calls", synth.scaled(synth.LLAMA, 262145, n_kv_heads=1, n_q_heads=1, head_dim=64), 0.05),
]


@pytest.mark.parametrize("name,w,ratio", CASES, ids=[c[0] for c in CASES])
def test_deviation_topk_equals_the_two_calls(name, w, ratio):
    say(f"deviation_topk {name}")
    lay = synth.make_layer(w, with_q=False)
    n_reused = int(lay["reused"].sum())
    k = max(1, min(w.n_ctx, synth.recompute_budget(n_reused, ratio))) if n_reused else 1
    sc, idx = fused_and_separate(w, lay, k)
    # against the oracle's scores: 1e-5, and the same candidate mask
    _, _, sc_ref = oracle.deviation(lay["v_fresh"], lay["v_cache"], reused=lay["reused"])
    fin = np.isfinite(sc_ref)
    assert np.array_equal(np.isfinite(sc), fin)
    np.testing.assert_allclose(sc[fin], sc_ref[fin], rtol=1e-5)
    # weighted, key+value mode, and without the score output
    alpha = synth.synthetic_alpha(w)
    fused_and_separate(w, lay, k, alpha=alpha, mode=B.SCORE_KV)
    fused_and_separate(w, lay, k, alpha=alpha, with_score=not (12288 < w.n_ctx <= 262144))


def test_deviation_topk_ties_and_non_candidates():
    """Thresholds inside ties, all scores equal (every key in one bin: the candidates do not fit the
    LDS list and are read from their segments instead), more entries asked for than finite scores
    (the list is completed with non-candidates, lowest indices first), k = n, no mask."""
    w = synth.scaled(synth.LLAMA, 20000, span_mean=64.0, coverage=0.5)
    say("deviation_topk ties")
    lay = synth.make_layer(w, with_q=False)
    n = w.n_ctx
    # quantise the noise: cache = fresh + one of three fixed offsets on every reused token -> three score levels
    vf = lay["v_fresh"].float()
    level = torch.from_numpy(np.random.default_rng(3).integers(0, 3, n)).view(n, 1, 1).float()
    lay["v_cache"] = torch.where(lay["reused"].bool().view(n, 1, 1), vf + 0.25 * (level + 1.0), vf).to(torch.bfloat16)
    lay["v_fresh"] = vf.to(torch.bfloat16)
    n_reused = int(lay["reused"].sum())
    for k in (1, n_reused // 3, n_reused // 2, n_reused - 1, n_reused, n_reused + 1, n_reused + 777, n):
        sc, idx = fused_and_separate(w, lay, k)
        if k > n_reused:
            assert np.isneginf(sc[idx]).sum() == k - n_reused
    # all equal: cache = fresh + a constant everywhere, every token a candidate
    lay["v_cache"] = (vf + 0.5).to(torch.bfloat16)
    lay["v_fresh"] = vf.to(torch.bfloat16)
    for k in (1, 5000, n - 1, n):
        fused_and_separate(w, lay, k, reused=None)
    # zero deviation everywhere (score +0 for all candidates)
    lay["v_cache"] = lay["v_fresh"].clone()
    fused_and_separate(w, lay, 1234)


def test_deviation_topk_empty_and_zero_k():
    w = synth.scaled(synth.LLAMA, 13000)
    sh = B.shape_of(w)
    lay = synth.make_layer(w, with_q=False)
    g = {key: v.to(DEV) for key, v in lay.items()}
    n, hk = w.n_ctx, w.n_kv_heads
    dev_v, score = torch.empty((hk, n), device=DEV), torch.full((n,), float("nan"), device=DEV)
    B.kvs_deviation_topk(sh, n, None, g["v_fresh"], None, g["v_cache"], g["reused"], None, B.SCORE_V, None, dev_v, score, 0, None)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(score).any())                    # k = 0: the scores are still produced
    B.kvs_deviation_topk(sh, 0, None, None, None, None, None, None, B.SCORE_V, None, None, None, 0, None)
    with pytest.raises(B.KvsError):
        B.kvs_deviation_topk(sh, n, None, g["v_fresh"], None, g["v_cache"], None, None, B.SCORE_V, None, None, score, n + 1,
                             torch.empty(1, dtype=torch.int32, device=DEV))
    # and the call after these still finds a clean histogram
    fused_and_separate(w, lay, 100)
