"""Pins for the oracle's Huffman code (Sec. IV-A (ii); optimality as cited in Sec. II-E)."""
import heapq
import itertools
import math
import os

import numpy as np
import pytest

from oracle import co3_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def check_prefix_free_and_kraft(lens, codes):
    act = [(int(l), int(c)) for l, c in zip(lens, codes) if l]
    strs = [format(c, "b").zfill(l) for l, c in act]
    for a, b in itertools.permutations(strs, 2):
        assert not b.startswith(a)
    if len(act) >= 2:
        Lmax = max(l for l, _ in act)
        assert sum(1 << (Lmax - l) for l, _ in act) == 1 << Lmax      # Kraft equality, exactly
    return strs


def test_golden_tie_cases():
    for line in open(os.path.join(GOLD, "huffman_ties.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w, l, c = [part.split() for part in line.split("|")]
        lens, codes = orc.codebook(np.array([int(x) for x in w], np.uint64))
        assert lens.tolist() == [int(x) for x in l], line
        got = [format(int(cd), "b").zfill(int(ln)) if ln else "-" for ln, cd in zip(lens, codes)]
        assert got == c, line


def bruteforce_min_cost(w):
    """Minimum of sum w_i l_i over all length vectors satisfying Kraft's inequality."""
    n = len(w)
    best = None
    for ls in itertools.product(range(1, n), repeat=n):
        if sum(2.0 ** -l for l in ls) <= 1.0:
            cost = sum(wi * li for wi, li in zip(w, ls))
            best = cost if best is None else min(best, cost)
    return best


@pytest.mark.parametrize("n", [2, 3, 4, 5, 6, 7])
def test_optimal_by_bruteforce(n):
    rng = np.random.default_rng(n)
    for trial in range(6 if n < 7 else 2):
        w = rng.integers(1, 12 if trial % 2 else 1000, n)
        lens, codes = orc.codebook(w.astype(np.uint64))
        check_prefix_free_and_kraft(lens, codes)
        assert int((w * lens).sum()) == bruteforce_min_cost(w.tolist())


def heap_cost(w):
    """Huffman cost as the sum of all merged weights (heapq; a different route to the cost)."""
    h = [int(x) for x in w if x > 0]
    heapq.heapify(h)
    cost = 0
    while len(h) > 1:
        a, b = heapq.heappop(h), heapq.heappop(h)
        cost += a + b
        heapq.heappush(h, a + b)
    return cost


@pytest.mark.parametrize("A", [16, 64, 256])
def test_cost_entropy_and_structure(A):
    rng = np.random.default_rng(A)
    for kind in range(6):
        if kind == 0:
            w = rng.integers(0, 1000, A)
        elif kind == 1:
            w = (rng.pareto(0.7, A) * 50).astype(np.int64)
        elif kind == 2:
            w = rng.integers(1, 3, A)
        elif kind == 3:
            w = np.zeros(A, np.int64); w[rng.choice(A, 5, replace=False)] = rng.integers(1, 10 ** 9, 5)
        elif kind == 4:
            w = (np.exp(-np.arange(A) / 3.0) * 4e9).astype(np.int64)
        else:
            w = rng.integers(1, 2 ** 40, A)
        w = w.astype(np.uint64)
        if (w > 0).sum() < 2:
            w[:2] = 1
        lens, codes = orc.codebook(w)
        assert np.all((lens > 0) == (w > 0))
        check_prefix_free_and_kraft(lens, codes)
        wf = w.astype(np.float64)
        cost = int(sum(int(a) * int(b) for a, b in zip(w, lens)))
        assert cost == heap_cost(w)
        p = wf[wf > 0] / wf.sum()
        H = -(p * np.log2(p)).sum()
        Lbar = cost / float(wf.sum())
        assert H - 1e-9 <= Lbar < H + 1
        # canonical: codes increase with (length, symbol)
        order = sorted((int(l), s) for s, l in enumerate(lens) if l)
        vals = [int(codes[s]) << (64 - l) if l < 64 else int(codes[s]) for l, s in order]
        assert vals == sorted(vals) and len(set(vals)) == len(vals)


def test_closed_forms():
    # dyadic probabilities: l = -log2 p
    w = np.array([8, 4, 2, 1, 1], np.uint64)
    assert orc.huffman_lengths(w).tolist() == [1, 2, 3, 4, 4]
    # uniform over 2^k symbols: all lengths k
    for k in (1, 4, 8):
        assert set(orc.huffman_lengths(np.full(1 << k, 7, np.uint64)).tolist()) == {k}
    # Fibonacci weights give the deepest tree: depths n-1, n-1, n-2, ..., 1
    fib = [1, 1]
    while len(fib) < 40:
        fib.append(fib[-1] + fib[-2])
    lens = orc.huffman_lengths(np.array(fib, np.uint64)).tolist()
    assert lens == [39, 39] + list(range(38, 0, -1))
    # weights 1, 1, 2, 4, ..., 2^62: depth 64 is the longest supported length
    w = np.array([1] + [1 << i for i in range(0, 63)], np.uint64)
    lens = orc.huffman_lengths(w).tolist()
    assert max(lens) == 63 and lens[0] == 63 and lens[-1] == 1
    codes = orc.canonical_codes(np.array(lens, np.uint8))
    check_prefix_free_and_kraft(lens, codes)


def test_too_deep_is_an_error():
    # 66 Fibonacci weights would need a 65-bit code
    fib = [1, 1]
    while len(fib) < 67:
        fib.append(fib[-1] + fib[-2])
    with pytest.raises(ValueError):
        orc.huffman_lengths(np.array(fib, np.uint64))


def test_degenerate_alphabets():
    assert orc.huffman_lengths(np.zeros(16, np.uint64)).tolist() == [0] * 16
    l, c = orc.codebook(np.array([0, 0, 9, 0], np.uint64))
    assert l.tolist() == [0, 0, 1, 0] and c.tolist() == [0, 0, 0, 0]
