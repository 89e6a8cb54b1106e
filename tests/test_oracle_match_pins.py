"""Pins for the oracle's token matcher, window hash and scheduler (App. E Alg. 3 and Eq. (7); Sec. 4.3 Alg. 2).

None of these re-runs the oracle's own procedure: the hash is pinned by worked values, closed
forms and exact integer arithmetic on Python integers; the matcher by a worked example, by
special cases whose answer is known without running anything, by a brute-force statement of what
the sequential procedure must end up with (for every target position, the earliest candidate
window -- then the earliest target window -- whose stretch of equal tokens reaches it), and by
inputs assembled from known pieces; the scheduler by numpy's stable sort.
"""
import numpy as np
import pytest

import oracle
from paper_2503_16525_amd import synth


def test_hash_worked_values():
    # base 10 reads the window as a decimal number
    assert oracle.window_hash([1, 2, 3, 4], 3, 10, 1000).tolist() == [123, 234]
    assert oracle.window_hash([1, 2, 3, 4], 3, 10, 100).tolist() == [23, 34]
    assert oracle.window_hash([7, 7, 7], 1, 12345, 5).tolist() == [2, 2, 2]          # w = 1: the token itself, mod m
    assert oracle.window_hash([9, 8, 7], 4, 10, 1000).tolist() == []                 # no window fits
    assert oracle.window_hash([5, 6, 7, 8], 2, 31, 1).tolist() == [0, 0, 0]          # m = 1


def test_hash_closed_form_equal_tokens():
    # a window of w equal tokens t: t (b^w - 1) / (b - 1)
    for (t, w, b, m) in ((3, 16, 257, 4294967291), (100000, 32, 1000003, 2147483647), (1, 5, 2, 1000)):
        want = (t * (b ** w - 1) // (b - 1)) % m
        assert oracle.window_hash([t] * (w + 3), w, b, m).tolist() == [want] * 4


def test_hash_exact_integers_and_rolling_identity():
    rng = np.random.default_rng(5)
    for (w, b, m) in ((8, 1000003, 4294967291), (16, 4294967295, 4294967295), (3, 2, 7)):
        t = rng.integers(0, 2 ** 31 - 1, size=40).tolist()
        h = oracle.window_hash(t, w, b, m).tolist()
        for i in (0, 7, len(t) - w):
            assert h[i] == sum(int(t[i + x]) * b ** (w - 1 - x) for x in range(w)) % m
        for i in range(len(t) - w):    # H(i+1) = H(i) b - t_i b^w + t_(i+w)
            assert h[i + 1] == (h[i] * b - t[i] * b ** w + t[i + w]) % m


def test_match_worked_example():
    # w = 3.  Candidate window 0 = (1,2,3) is target window 5: pairs (5,0) (6,1) (7,2).  Candidate
    # windows 1 and 2 occur nowhere.  Candidate window 3 = (5,6,7) is target window 0 and the
    # tokens keep agreeing for one more: (0,3) (1,4) (2,5) (3,6).  Candidate window 4 = (6,7,8) is
    # target window 1, whose positions are taken already.
    tm, cm = oracle.match_tokens([5, 6, 7, 8, 9, 1, 2, 3], [1, 2, 3, 5, 6, 7, 8], 3, 31, 1000003)
    assert tm.tolist() == [5, 6, 7, 0, 1, 2, 3]
    assert cm.tolist() == [0, 1, 2, 3, 4, 5, 6]


def test_match_special_cases():
    rng = np.random.default_rng(11)
    t = rng.permutation(500)[:300].tolist()           # all tokens different
    tm, cm = oracle.match_tokens(t, t, 8, 1000003, 4294967291)
    assert tm.tolist() == list(range(300)) and cm.tolist() == list(range(300))
    # a candidate that holds the target after 17 other tokens
    tm, cm = oracle.match_tokens(t, list(range(1000, 1017)) + t, 8, 1000003, 4294967291)
    assert tm.tolist() == list(range(300)) and cm.tolist() == list(range(17, 317))
    # nothing in common; sequences shorter than the window; empty sequences
    assert oracle.match_tokens(t, [x + 1000 for x in t], 8, 1000003, 4294967291)[0].size == 0
    assert oracle.match_tokens(t[:7], t[:7], 8, 1000003, 4294967291)[0].size == 0
    assert oracle.match_tokens([], t, 8, 1000003, 4294967291)[0].size == 0
    assert oracle.match_tokens(t, [], 8, 1000003, 4294967291)[0].size == 0
    # a common stretch shorter than the window is not found (no window of it exists in both)
    tm, _ = oracle.match_tokens(t[:100], [900, 901] + t[40:47] + [902, 903, 904], 8, 1000003, 4294967291)
    assert tm.size == 0
    # ... and one of exactly the window's length is
    tm, cm = oracle.match_tokens(t[:100], [900, 901] + t[40:48] + [902, 903, 904], 8, 1000003, 4294967291)
    assert tm.tolist() == list(range(40, 48)) and cm.tolist() == list(range(2, 10))


def brute_force(target, candidate, w, b, m):
    """What Alg. 3 must end with, stated without its loop order: target position p is matched iff
    some pair of window starts (i, j) with equal hashes has equal tokens from (i, j) up to (p, j+p-i);
    its partner is j+p-i for the smallest such (j, i) in lexicographic order; pairs are listed by
    (j, i, p)."""
    nt, nc = len(target), len(candidate)
    H = lambda s, i: sum(int(s[i + x]) * b ** (w - 1 - x) for x in range(w)) % m
    ht = [H(target, i) for i in range(nt - w + 1)]
    hc = [H(candidate, j) for j in range(nc - w + 1)]
    best = {}
    for p in range(nt):
        for j in range(len(hc)):
            found = None
            for i in range(min(p, len(ht) - 1) + 1):
                if ht[i] != hc[j] or j + p - i >= nc:
                    continue
                if all(target[i + k] == candidate[j + k] for k in range(p - i + 1)):
                    found = i
                    break
            if found is not None:
                best[p] = (j, found)
                break
    pairs = sorted((j, i, p) for p, (j, i) in best.items())
    return [p for (_, _, p) in pairs], [j + p - i for (j, i, p) in pairs]


@pytest.mark.parametrize("seed", range(12))
def test_match_equals_brute_force_statement(seed):
    rng = np.random.default_rng(100 + seed)
    vocab = (2, 3, 5, 50)[seed % 4]                     # tiny vocabularies: many repeats and overlapping stretches
    w = (1, 2, 3, 4)[(seed // 4) % 4]
    m = (1, 3, 7, 4294967291)[seed % 4 if seed < 8 else 3]   # tiny moduli: windows that differ collide
    b = (31, 2, 1000003)[seed % 3]
    nt, nc = int(rng.integers(w, 40)), int(rng.integers(w, 40))
    target = rng.integers(0, vocab, size=nt).tolist()
    candidate = rng.integers(0, vocab, size=nc).tolist()
    if seed % 2:                                         # plant a copied stretch
        L = min(nt, nc, 12)
        a, c = int(rng.integers(0, nt - L + 1)), int(rng.integers(0, nc - L + 1))
        target[a:a + L] = candidate[c:c + L]
    tm, cm = oracle.match_tokens(target, candidate, w, b, m)
    want_t, want_c = brute_force(target, candidate, w, b, m)
    assert tm.tolist() == want_t and cm.tolist() == want_c


def test_match_all_equal_tokens():
    # every window of both sequences is the same: candidate window 0 claims the target from each
    # target start in turn, so target position p ends up with candidate position 0 ... see the statement:
    # smallest j = 0, then smallest i = 0: partner of p is p while p < n_candidate, and beyond that
    # the smallest (j, i) that still reaches p
    tm, cm = oracle.match_tokens([4] * 10, [4] * 6, 3, 31, 1000003)
    want_t, want_c = brute_force([4] * 10, [4] * 6, 3, 31, 1000003)
    assert tm.tolist() == want_t and cm.tolist() == want_c
    assert sorted(tm.tolist()) == list(range(10))


def test_match_recovers_planted_spans():
    s = synth.make_token_streams(synth.scaled(synth.QWEN, 4096), seed=3, window=16)
    tm, cm = oracle.match_tokens(s["target"], s["candidate"], 16, 1000003, 4294967291)
    partner = np.full(s["target"].shape[0], -1, dtype=np.int64)
    partner[tm] = cm
    assert np.array_equal(s["target"][tm], s["candidate"][cm])           # matched tokens are equal tokens
    planted = s["source"] >= 0
    long_enough = planted & (s["span_len"] >= 16)
    assert np.all(partner[long_enough] >= 0)                             # every copied stretch of >= w tokens is found
    # the candidate's tokens are all different, so the partner is the position the stretch was copied from
    assert np.array_equal(partner[long_enough], s["source"][long_enough])
    assert not np.any(partner[~planted] >= 0)                            # fresh tokens come from a disjoint range
    assert len(set(tm.tolist())) == tm.size                              # a target position is matched once


def test_schedule_is_a_stable_descending_sort():
    assert oracle.schedule([0.1, 0.9, 0.5, 0.9]).tolist() == [1, 3, 2, 0]
    rng = np.random.default_rng(2)
    h = np.round(rng.random(200), 1).astype(np.float32)                  # many equal rates
    assert oracle.schedule(h).tolist() == np.argsort(-h, kind="stable").tolist()
    assert oracle.schedule([]).size == 0
