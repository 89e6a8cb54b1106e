"""Seeded synthetic workloads shaped like the paper's 7-9B-model layers.

This module only draws random inputs (span structure, fresh Q/K/V, the noisy
reused cache).  It contains none of the method's arithmetic: no deviation, no
scoring, no selection, no attention.  Both the CPU oracle's tests and the HIP
path's tests/bench take their inputs from here so that the two sides see the
same bits.

The paper evaluates on Qwen2.5-7B / Llama3.1-8B / Yi1.5-9B with real prompts
(experimental setup, Sec. 5.1); neither the weights nor the datasets are
available, so every tensor here is a seeded stand-in with the head counts,
head size and context lengths of those models.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np
import torch

BASE_SEED = 20250316


@dataclass(frozen=True)
class Workload:
    name: str
    index: int            # position in the benchmark's config list (seed offset)
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_ctx: int
    dtype: str            # "f32" | "bf16"
    span_mean: float      # mean reused-span length (geometric); unused when n_spans > 0
    coverage: float       # expected fraction of the context that is reused
    sigma_mu: float       # per-token noise std is lognormal(mu, s)
    sigma_s: float
    ratios: Tuple[float, ...]   # recompute ratios, as a fraction of reused tokens
    n_spans: int = 0      # >0: exactly this many spans with lengths U{span_lo..span_hi}
    span_lo: int = 0
    span_hi: int = 0
    hidden: int = 0       # >0: Q/K/V may be produced by random projections from this width

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


TINY = Workload("tiny-f32", 0, 4, 4, 64, 512, "f32", 0.0, 0.0, -3.0, 1.0, (0.15,),
                n_spans=4, span_lo=32, span_hi=128)
QWEN = Workload("qwen2.5-7b-layer", 1, 28, 4, 128, 8192, "bf16", 256.0, 0.80, -3.0, 1.5, (0.10,))
LLAMA = Workload("llama3.1-8b-layer", 2, 32, 8, 128, 32768, "bf16", 512.0, 0.90, -3.0, 1.5,
                 (0.05, 0.15, 0.30), hidden=4096)
YI = Workload("yi1.5-9b-layer", 3, 32, 4, 128, 131072, "bf16", 1024.0, 0.95, -3.0, 1.5, (0.10,))
DECODE = Workload("llama3.1-8b-decode", 4, 32, 8, 128, 0, "bf16", 0.0, 1.0, -3.0, 1.5, (0.02,))

WORKLOADS: Dict[str, Workload] = {w.name: w for w in (TINY, QWEN, LLAMA, YI, DECODE)}


def scaled(w: Workload, n_ctx: int, name: Optional[str] = None, **kw) -> Workload:
    """Same shape family at another context length (used for mid-size test cases)."""
    d = dict(w.__dict__)
    d.update(n_ctx=n_ctx, name=name or f"{w.name}@{n_ctx}")
    d.update(kw)
    return Workload(**d)


def layer_seed(w: Workload, layer: int = 0, salt: int = 0) -> int:
    return BASE_SEED + 1000 * w.index + layer + 1_000_003 * salt


def _np_rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=seed))


def make_spans(w: Workload, seed: int) -> np.ndarray:
    """uint8[n_ctx], 1 where the token's K/V comes from another request's cache."""
    n = w.n_ctx
    rng = _np_rng(seed ^ 0x5EED5)
    reused = np.zeros(n, dtype=np.uint8)
    if w.n_spans > 0:
        # exactly n_spans non-touching spans: draw lengths, then spread the slack as gaps >= 1
        for _ in range(1000):
            lens = rng.integers(w.span_lo, w.span_hi + 1, size=w.n_spans)
            slack = n - int(lens.sum()) - (w.n_spans + 1)
            if slack >= 0:
                break
        else:
            raise ValueError("spans do not fit the context")
        cuts = np.sort(rng.integers(0, slack + 1, size=w.n_spans + 1))
        extra = np.diff(np.concatenate([[0], cuts]))          # n_spans+1 nonneg ints, sum <= slack
        pos = 0
        for s in range(w.n_spans):
            pos += 1 + int(extra[s])
            reused[pos:pos + lens[s]] = 1
            pos += int(lens[s])
        return reused
    if w.coverage >= 1.0:
        reused[:] = 1
        return reused
    gap_mean = w.span_mean * (1.0 - w.coverage) / w.coverage
    pos = 0
    # start with a fresh gap (the request's own system prompt / new text)
    while pos < n:
        gap = int(rng.geometric(1.0 / max(gap_mean, 1.0)))
        pos += gap
        if pos >= n:
            break
        span = int(rng.geometric(1.0 / w.span_mean))
        reused[pos:pos + span] = 1
        pos += span
    return reused


def _randn(shape, gen: torch.Generator, device) -> torch.Tensor:
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32)


def make_layer(w: Workload, layer: int = 0, device: str = "cpu", projected: bool = False,
               salt: int = 0, with_q: bool = True) -> Dict[str, torch.Tensor]:
    """One attention layer's inputs.

    Returns q [N,Hq,d] (pre-scaled by 1/sqrt(d); use scale=1), k_fresh, v_fresh,
    k_cache, v_cache [N,Hkv,d] in the workload dtype, reused uint8[N] and
    sigma float32[N] (the per-token noise std that was applied).
    """
    seed = layer_seed(w, layer, salt)
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    n, hq, hkv, d = w.n_ctx, w.n_q_heads, w.n_kv_heads, w.head_dim
    dt = w.torch_dtype
    out: Dict[str, torch.Tensor] = {}
    if projected:
        if w.hidden <= 0:
            raise ValueError("workload has no hidden size for projections")
        x = _randn((n, w.hidden), gen, dev).to(dt)
        std = 1.0 / math.sqrt(w.hidden)
        wq = (_randn((w.hidden, hq * d), gen, dev) * std).to(dt)
        wk = (_randn((w.hidden, hkv * d), gen, dev) * std).to(dt)
        wv = (_randn((w.hidden, hkv * d), gen, dev) * std).to(dt)
        if with_q:
            out["q"] = ((x @ wq).float() / math.sqrt(d)).to(dt).view(n, hq, d)
        k32 = (x @ wk).float().view(n, hkv, d)
        v32 = (x @ wv).float().view(n, hkv, d)
        del x, wq, wk, wv
    else:
        if with_q:
            out["q"] = (_randn((n, hq, d), gen, dev) / math.sqrt(d)).to(dt)
        k32 = _randn((n, hkv, d), gen, dev)
        v32 = _randn((n, hkv, d), gen, dev)
    k_fresh = k32.to(dt)
    v_fresh = v32.to(dt)
    reused_np = make_spans(w, seed)
    reused = torch.from_numpy(reused_np).to(dev)
    z = _randn((n,), gen, dev)
    sigma = torch.exp(w.sigma_mu + w.sigma_s * z)
    m = reused.bool().view(n, 1, 1)
    s3 = sigma.view(n, 1, 1)
    # the cache holds what another request computed: the fresh value plus per-token noise,
    # rounded to the storage dtype; misses hold the fresh value itself
    k_cache = torch.where(m, (k_fresh.float() + s3 * _randn((n, hkv, d), gen, dev)).to(dt), k_fresh)
    v_cache = torch.where(m, (v_fresh.float() + s3 * _randn((n, hkv, d), gen, dev)).to(dt), v_fresh)
    out.update(k_fresh=k_fresh, v_fresh=v_fresh, k_cache=k_cache, v_cache=v_cache,
               reused=reused, sigma=sigma)
    return out


def recompute_budget(n_reused: int, ratio: float) -> int:
    """k = ceil(ratio * number of reused tokens), the caller-side reading of 'top-r%'."""
    return int(math.ceil(ratio * n_reused - 1e-9))


def synthetic_alpha(w: Workload, layer: int = 0, device: str = "cpu") -> torch.Tensor:
    """A stand-in attention column-mass profile [Hkv, N] for contexts too long for the exact
    O(N^2) computation: the harmonic tail that uniform causal attention would give, times a
    seeded jitter in [1, 2), times the group size."""
    n = w.n_ctx
    gen = torch.Generator(device=torch.device(device))
    gen.manual_seed(layer_seed(w, layer, salt=7))
    inv = 1.0 / torch.arange(1, n + 1, dtype=torch.float64)
    tail = torch.flip(torch.cumsum(torch.flip(inv, [0]), 0), [0]).float().to(device)
    u = torch.rand((w.n_kv_heads, n), generator=gen, device=device)
    return (w.group * tail.view(1, n) * (1.0 + u)).contiguous()


def make_decode_batch(w: Workload, batch: int, len_lo: int, len_hi: int, n_steps: int,
                      device: str = "cpu", salt: int = 0) -> Dict[str, torch.Tensor]:
    """A ragged batch of fully reused contexts for the decode stage.

    Request b owns rows [ctx_off[b], ctx_off[b] + ctx_len[b] + n_steps) of the packed cache
    (slack for the tokens appended during decoding).  Returns k_fresh/v_fresh/k_cache/v_cache
    [rows,Hkv,d], reused uint8[rows] (1 on the initial context, 0 on the slack), ctx_off and
    ctx_len as int64 numpy arrays, and per-step new-token tensors q_new [S,B,Hq,d] (pre-scaled),
    k_new/v_new [S,B,Hkv,d].
    """
    seed = layer_seed(w, 0, salt)
    rng = _np_rng(seed ^ 0xDEC0DE)
    lens = rng.integers(len_lo, len_hi + 1, size=batch).astype(np.int64)
    cap = lens + n_steps
    off = np.concatenate([[0], np.cumsum(cap)[:-1]]).astype(np.int64)
    rows = int(cap.sum())
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    hq, hkv, d = w.n_q_heads, w.n_kv_heads, w.head_dim
    dt = w.torch_dtype
    k_fresh = _randn((rows, hkv, d), gen, dev).to(dt)
    v_fresh = _randn((rows, hkv, d), gen, dev).to(dt)
    reused_np = np.zeros(rows, dtype=np.uint8)
    for b in range(batch):
        reused_np[off[b]:off[b] + lens[b]] = 1
    reused = torch.from_numpy(reused_np).to(dev)
    sigma = torch.exp(w.sigma_mu + w.sigma_s * _randn((rows,), gen, dev))
    m = reused.bool().view(rows, 1, 1)
    s3 = sigma.view(rows, 1, 1)
    k_cache = torch.where(m, (k_fresh.float() + s3 * _randn((rows, hkv, d), gen, dev)).to(dt), k_fresh)
    v_cache = torch.where(m, (v_fresh.float() + s3 * _randn((rows, hkv, d), gen, dev)).to(dt), v_fresh)
    q_new = (_randn((n_steps, batch, hq, d), gen, dev) / math.sqrt(d)).to(dt)
    k_new = _randn((n_steps, batch, hkv, d), gen, dev).to(dt)
    v_new = _randn((n_steps, batch, hkv, d), gen, dev).to(dt)
    return dict(k_fresh=k_fresh, v_fresh=v_fresh, k_cache=k_cache, v_cache=v_cache, reused=reused,
                ctx_off=off, ctx_len=lens, q_new=q_new, k_new=k_new, v_new=v_new)


def make_token_streams(w: Workload, seed: int = 0, window: int = 16, unique_candidate: bool = True,
                       vocab: int = 128256) -> Dict[str, np.ndarray]:
    """A target token sequence assembled from stretches of an earlier request (the candidate) and fresh text.

    The reused stretches are those of ``make_spans`` (the same span structure the K/V workloads use);
    each is copied from a random place in the candidate, the rest of the target is fresh.  With
    ``unique_candidate`` the candidate's tokens are all different and the fresh tokens come from a
    disjoint range, so the only common stretches are the copied ones and each has one source; otherwise
    both are drawn from one Zipf-like distribution over ``vocab`` ids, where frequent tokens repeat and
    short accidental stretches occur, as in text.

    Returns int32 ``target`` [n_ctx], ``candidate`` [n_ctx], and per target position ``source`` (the
    candidate position it was copied from, -1 for fresh text) and ``span_len`` (length of the copied
    stretch it belongs to, 0 for fresh text).
    """
    n = w.n_ctx
    rng = _np_rng(layer_seed(w, 0, salt=seed) ^ 0x70C3)
    if unique_candidate:
        candidate = rng.permutation(2 * n)[:n].astype(np.int32)
        fresh = (2 * n + rng.integers(0, n, size=n)).astype(np.int32)
    else:
        ranks = np.minimum(rng.zipf(1.2, size=2 * n), vocab) - 1
        ids = rng.permutation(vocab)
        candidate = ids[ranks[:n]].astype(np.int32)
        fresh = ids[ranks[n:]].astype(np.int32)
    reused = make_spans(w, layer_seed(w, 0, salt=seed))
    target = fresh.copy()
    source = np.full(n, -1, dtype=np.int64)
    span_len = np.zeros(n, dtype=np.int64)
    edges = np.flatnonzero(np.diff(np.concatenate([[0], reused, [0]])))
    for a, e in zip(edges[0::2], edges[1::2]):
        L = int(e - a)
        c = int(rng.integers(0, n - L + 1))
        target[a:e] = candidate[c:c + L]
        source[a:e] = np.arange(c, c + L)
        span_len[a:e] = L
    return dict(target=target, candidate=candidate, source=source, span_len=span_len)


def make_rope_table(n_positions: int, head_dim: int, theta: float = 500000.0) -> np.ndarray:
    """fp32 [n_positions, head_dim/2, 2]: cos and sin of position * theta^(-2c/head_dim), the rotary factors
    of the Llama / Qwen / Yi families (angles taken in fp64, rounded once).  An input table, as serving
    stacks keep it; the projection call and the oracle both read it."""
    half = head_dim // 2
    inv_freq = theta ** (-np.arange(half, dtype=np.float64) * 2.0 / head_dim)
    ang = np.arange(n_positions, dtype=np.float64)[:, None] * inv_freq[None, :]
    return np.stack([np.cos(ang), np.sin(ang)], axis=-1).astype(np.float32)


def make_projection(w: Workload, hidden: int, layer: int = 0, device: str = "cpu"):
    """Hidden states [n_ctx, hidden] ~ N(0,1) and a fused QKV weight [(H_q + 2 H_kv) d, hidden] ~ N(0, 1/hidden)
    in the workload's dtype (the marginals of the projected Q/K/V are those of the other generators)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(layer_seed(w, layer, salt=23))
    x = torch.randn((w.n_ctx, hidden), generator=gen, device=device).to(w.torch_dtype)
    feats = (w.n_q_heads + 2 * w.n_kv_heads) * w.head_dim
    wt = (torch.randn((feats, hidden), generator=gen, device=device) / math.sqrt(hidden)).to(w.torch_dtype)
    return x, wt
