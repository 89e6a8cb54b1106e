"""kvs_select_topk_static, the entry point for callers that cannot allocate device memory: same
results as kvs_select_topk given a workspace, on two calls in a row (the second on a smaller
input, so whatever the first left in the library's scratch is still there), through the C ABI."""
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2503_16525_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def both_ways(scores_np, row_off, k_row):
    scores = torch.from_numpy(scores_np).to(DEV)
    total = int(np.sum(k_row))
    sh = B.make_shape(8, 8, 128, B.BF16)
    ws = torch.empty(B.kvs_workspace_size("select_topk", sh, len(k_row), len(scores_np)), dtype=torch.uint8, device=DEV)
    want = torch.full((total,), -1, dtype=torch.int32, device=DEV)
    B.kvs_select_topk(scores, row_off, k_row, want, ws)
    got = torch.full((total,), -2, dtype=torch.int32, device=DEV)
    B.kvs_select_topk_static(scores, row_off, k_row, got)
    torch.cuda.synchronize()
    return got.cpu().numpy(), want.cpu().numpy()


def test_select_topk_static_matches_the_workspace_call_twice_in_a_row():
    B.kvs_select_topk_static(None, [0], [], None)        # n_rows = 0: only looks the scratch address up
    rng = np.random.default_rng(12)
    # first call: a 300k-score row (ten parts, a tie cut across parts), a short row and a 70k one
    big = rng.standard_normal(300_000).astype(np.float32)
    big[rng.integers(0, 300_000, 40_000)] = 0.75          # a large tie at what will be the threshold
    short = rng.standard_normal(5_000).astype(np.float32)
    mid = np.abs(rng.standard_normal(70_000)).astype(np.float32)
    scores = np.concatenate([big, short, mid])
    row_off = [0, 300_000, 305_000, 375_000]
    k_row = [int((big > 0.75).sum()) + 1234, 700, 7_000]
    say("no-alloc select: 300k + 5k + 70k rows")
    got, want = both_ways(scores, row_off, k_row)
    np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(got, oracle.select_topk(scores, row_off, k_row))
    # second call, smaller: one 60k-score row (two parts) after the scratch has been used
    small = rng.standard_normal(60_001).astype(np.float32)
    say("no-alloc select: 60k row")
    got2, want2 = both_ways(small, [0, 60_001], [6_000])
    np.testing.assert_array_equal(got2, want2)
    np.testing.assert_array_equal(got2, oracle.select_topk(small, [0, 60_001], [6_000]))


def test_select_topk_static_rejects_rows_beyond_its_scratch():
    scores = torch.zeros(8, device=DEV)
    idx = torch.empty(1, dtype=torch.int32, device=DEV)
    with pytest.raises(B.KvsError) as e:
        B.kvs_select_topk_static(scores, [0, (1 << 20) + 1], [1], idx)     # rejected on the host, nothing is read
    assert e.value.status == B.EINVAL and "scratch" in str(e.value)
