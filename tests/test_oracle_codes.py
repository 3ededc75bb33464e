"""Pins for the oracle's Huffman code construction (length-limited, canonical)."""
import heapq
import itertools
import math
import os

import numpy as np
import pytest

from oracle import zc_oracle as o

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _golden():
    for line in open(os.path.join(GOLD, "codes.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            L, f, ln, cost, codes = [p.strip() for p in line.split("|")]
            yield int(L), [int(v) for v in f.split()], [int(v) for v in ln.split()], int(cost), codes.split()


def kraft16(lengths):
    return sum(1 << (16 - int(l)) for l in lengths if l)


def entropy(freq):
    f = np.asarray([v for v in freq if v], float)
    p = f / f.sum()
    return float(-(p * np.log2(p)).sum())


def brute_force_cost(freq, L):
    """Cheapest complete prefix code with all lengths <= L, by enumeration.  The optimum
    gives non-increasing lengths to non-decreasing weights, so it is enough to try
    non-increasing length vectors on the sorted weights."""
    w = sorted(v for v in freq if v)
    n, best = len(w), None
    for ln in itertools.combinations_with_replacement(range(L, 0, -1), n):
        if sum(1 << (L - l) for l in ln) == 1 << L:
            c = sum(a * b for a, b in zip(w, ln))
            best = c if best is None else min(best, c)
    return best


def heap_huffman_cost(freq):
    """Textbook Huffman: the sum of all internal node weights equals sum(f*len)."""
    h = [v for v in freq if v]
    heapq.heapify(h)
    cost = 0
    while len(h) > 1:
        a, b = heapq.heappop(h), heapq.heappop(h)
        cost += a + b
        heapq.heappush(h, a + b)
    return cost


def test_golden_codes():
    n = 0
    for L, f, ln, cost, codes in _golden():
        got = o.code_lengths(f, L)
        assert got.tolist() == ln, (L, f)
        assert sum(a * b for a, b in zip(f, ln)) == cost
        assert brute_force_cost(f, L) == cost, (L, f)       # the hand-worked cost is optimal
        cc = o.canonical_codes(got)
        for v, text in enumerate(codes):
            if text == "-":
                assert got[v] == 0
            else:
                assert len(text) == got[v] and int(text, 2) == cc[v], (L, f, v)
        n += 1
    assert n >= 8


def test_brute_force_optimal_small_alphabets():
    rng = np.random.default_rng(3)
    for trial in range(400):
        n = int(rng.integers(2, 9))
        kind = trial % 4
        if kind == 0:
            f = rng.integers(1, 10, n)
        elif kind == 1:
            f = rng.integers(1, 1000, n)
        elif kind == 2:
            f = np.floor(np.exp2(rng.uniform(0, 12, n))).astype(int)    # steep: limits bind
        else:
            f = np.array([rng.integers(1, 4)] * n)                       # many ties
        f = [int(v) for v in f]
        for L in range(max(1, math.ceil(math.log2(n))), 8):
            ln = o.code_lengths(f, L)
            assert ln.max() <= L and ln.min() >= 1
            assert kraft16(ln) == 65536
            assert sum(a * int(b) for a, b in zip(f, ln)) == brute_force_cost(f, L), (f, L)


def test_matches_heap_huffman_when_limit_is_slack():
    rng = np.random.default_rng(4)
    for trial in range(200):
        n = int(rng.integers(2, 257))
        f = rng.integers(1, 1 << int(rng.integers(1, 9)), n).tolist()
        ln = o.code_lengths(f, 16)
        if ln.max() < 16:           # limit did not bind -> cost must equal plain Huffman
            assert sum(a * int(b) for a, b in zip(f, ln)) == heap_huffman_cost(f)
        else:
            assert sum(a * int(b) for a, b in zip(f, ln)) >= heap_huffman_cost(f)
        assert kraft16(ln) == 65536


def test_kraft_entropy_bounds_and_limit():
    rng = np.random.default_rng(5)
    for trial in range(300):
        A = [4, 16, 256][trial % 3]
        f = np.floor(np.exp2(rng.uniform(0, 24, A)) * (rng.random(A) < 0.8)).astype(np.int64)
        if (f > 0).sum() < 2:
            continue
        na = int((f > 0).sum())
        for L in (16, 12, 8):
            if (1 << L) < na:
                continue
            ln = o.code_lengths(f.tolist(), L)
            assert np.array_equal(ln > 0, f > 0)
            assert ln.max() <= L
            assert kraft16(ln) == 65536
            mean = float((f * ln).sum()) / float(f.sum())
            H = entropy(f)
            assert mean >= H - 1e-9
            if ln.max() < L:
                assert mean < H + 1
            # limiting more can only cost more
        c16 = int((f * o.code_lengths(f.tolist(), 16)).sum())
        c12 = int((f * o.code_lengths(f.tolist(), 12)).sum())
        assert c12 >= c16


def test_special_histograms():
    assert o.code_lengths([1] * 16, 8).tolist() == [4] * 16          # uniform -> flat
    assert o.code_lengths([7] * 256, 16).tolist() == [8] * 256
    assert o.code_lengths([3, 3, 3, 3], 2).tolist() == [2] * 4
    assert o.code_lengths([0, 9, 0, 0], 8).tolist() == [0, 1, 0, 0]  # single symbol (stored CONST)
    assert o.code_lengths([0, 0, 0, 0], 8).tolist() == [0, 0, 0, 0]
    with pytest.raises(ValueError):
        o.code_lengths([1] * 9, 3)
    # dyadic weights: mean length equals the entropy
    f = [128, 64, 32, 16, 8, 4, 2, 1, 1]
    ln = o.code_lengths(f, 16)
    assert abs(sum(a * int(b) for a, b in zip(f, ln)) / sum(f) - entropy(f)) < 1e-12


def test_canonical_codes_are_prefix_free_and_ordered():
    rng = np.random.default_rng(6)
    for _ in range(50):
        f = np.floor(np.exp2(rng.uniform(0, 18, 64))).astype(int).tolist()
        ln = o.code_lengths(f, 12)
        cc = o.canonical_codes(ln)
        words = sorted((format(int(c), "b").zfill(int(l)), v) for v, (c, l) in enumerate(zip(cc, ln)))
        for (a, _), (b, _) in zip(words, words[1:]):
            assert not b.startswith(a)
        # ordered by (length, symbol): numeric order of left-aligned codes follows that order
        order = sorted(range(64), key=lambda v: (ln[v], v))
        aligned = [int(cc[v]) << (16 - int(ln[v])) for v in order]
        assert aligned == sorted(aligned) and aligned[0] == 0
