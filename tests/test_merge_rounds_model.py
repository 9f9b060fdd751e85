"""The device builders run the two-queue Huffman merge (Sec. IV-A (ii)) in rounds: every node that the
serial merge would take before any node it has yet to create is paired off at once.  This file restates
that schedule in plain Python and checks, without a GPU, that it gives the oracle's code lengths on tables
with many ties, one and two symbols, powers of two, Fibonacci weights and counts as a round produces them.
(The kernels themselves are compared with the oracle in tests/test_gpu_parity.py.)"""
import bisect

import numpy as np
import pytest

from oracle import co3_oracle as orc

NONE = (1 << 64) - 1


def lengths_by_rounds(w):
    A = len(w)
    act = sorted((int(w[s]), s) for s in range(A) if w[s] > 0)      # leaves by (weight, symbol)
    n = len(act)
    lens = np.zeros(A, np.uint8)
    if n == 0:
        return lens, 0
    if n == 1:
        lens[act[0][1]] = 1
        return lens, 0
    nw = [x[0] for x in act] + [None] * n                             # leaves, then internal nodes as created
    parent = [-1] * (2 * n)
    li, ii, made = 0, n, n                                            # next leaf, next internal node, next to create
    rounds = 0
    while (n - li) + (made - ii) > 1:
        c0 = nw[li] if li < n else NONE
        c1 = nw[li + 1] if li + 1 < n else NONE
        c2 = nw[ii] if ii < made else NONE
        c3 = nw[ii + 1] if ii + 1 < made else NONE
        m1 = min(c0, c2)
        m2 = min((c1, c2) if c0 < c2 else (c0, c3))                   # the two lightest of two sorted pairs
        T = m1 + m2
        assert T < NONE
        lj = bisect.bisect_right(nw, T, li, n)                        # leaves of weight <= T
        bL, bI = lj - li, made - ii
        nb = bL + bI
        assert nb >= 2
        order = [None] * nb
        for e in range(nb):
            if e < bL:
                node = li + e
                r = e + (bisect.bisect_left(nw, nw[node], ii, made) - ii)     # lighter internal nodes
            else:
                node = ii + (e - bL)
                r = (e - bL) + (bisect.bisect_right(nw, nw[node], li, lj) - li)  # leaves that are not heavier
            assert order[r] is None
            order[r] = node
        for k in range(nb // 2):
            a, b = order[2 * k], order[2 * k + 1]
            nw[made + k] = nw[a] + nw[b]
            parent[a] = parent[b] = made + k
        if nb & 1:   # the heaviest stays: the last internal node unless a leaf is heavier
            if bI > 0 and (bL == 0 or nw[made - 1] >= nw[lj - 1]):
                li, ii = lj, made - 1
            else:
                li, ii = lj - 1, made
        else:
            li, ii = lj, made
        made += nb // 2
        rounds += 1
    for i in range(n):
        d, p = 0, parent[i]
        while p >= 0:
            d, p = d + 1, parent[p]
        lens[act[i][1]] = d
    return lens, rounds


def tables(A, rng):
    yield rng.integers(0, 4, A)
    yield rng.integers(0, 1000, A)
    yield np.ones(A, np.int64)
    one = np.zeros(A, np.int64); one[A - 3] = 5
    yield one
    two = np.zeros(A, np.int64); two[0] = 7; two[A - 1] = 7
    yield two
    k = min(A, 40)
    path = np.zeros(A, np.int64); path[rng.choice(A, k, replace=False)] = [1 << int(i) for i in rng.permutation(k)]
    yield path
    yield np.floor(1e6 * np.exp(-np.arange(A) / (A / 20))).astype(np.int64)
    t = rng.integers(1, 6, A); t[rng.choice(A, A // 3, replace=False)] = 0
    yield t
    fib = np.zeros(A, np.int64); a, b = 1, 1
    for i in range(min(A, 60)):
        fib[i] = a; a, b = b, a + b
    yield fib


@pytest.mark.parametrize("A", [8, 16, 64, 256, 512, 4096])
def test_rounds_give_the_serial_merges_code_lengths(A):
    rng = np.random.default_rng(1700 + A)
    for rep in range(3 if A < 4096 else 1):
        for w in tables(A, rng):
            w = np.asarray(w, np.uint64)
            got, rounds = lengths_by_rounds(w)
            assert np.array_equal(got, orc.huffman_lengths(w))
            assert rounds <= max(1, int((w > 0).sum()) - 1)


def test_rounds_are_few_on_counts_and_many_on_a_path():
    A = 256
    counts = np.floor(4e8 * np.exp(-np.arange(A) / 12.0)).astype(np.uint64)
    _, r = lengths_by_rounds(counts)
    assert r <= 64                       # some tens of rounds for 200 and more active symbols
    path = np.zeros(A, np.uint64); path[:40] = [1 << i for i in range(40)]
    _, r = lengths_by_rounds(path)
    assert r == 39                       # one pair per round: the serial merge
