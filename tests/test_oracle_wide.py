"""Pins of the oracle's alphabets wider than one byte (symbols in 16-bit words; reading R17): the steps are
the byte path's, so the pins are the ones that do not depend on the symbol width, at formats of 9 to 12 bits:
nearest representative against a library cast (IEEE half is [1,5,10]; here [1,5,6] agrees with float16 rounded
to 6 mantissa bits for inputs where both roundings coincide, i.e. exact multiples), the exact-rational argmin on
grid points and midpoints, histogram = bincount, Huffman cost = heapq cost and Kraft equality, pack/unpack round
trip with a hand-checkable two-symbol stream, aggregate against exact rationals."""
import heapq
from fractions import Fraction

import numpy as np
import pytest

import co3_synth as syn
from oracle import co3_oracle as orc
from oracle import co3_round as oround


@pytest.mark.parametrize("E,M,bias", [(5, 6, 20), (4, 5, 14), (3, 5, 6), (5, 3, 18)])
def test_wide_conversion_is_the_exact_nearest(E, M, bias):
    mag = orc.grid(E, M, bias)
    assert mag.size == ((1 << E) - 1) << M
    rng = np.random.default_rng(E * 100 + M)
    mids = (mag[:-1] + mag[1:]) / 2
    pts = np.concatenate([mag, mids, np.nextafter(mids.astype(np.float32), np.float32(np.inf)),
                          np.nextafter(mids.astype(np.float32), np.float32(0))]).astype(np.float32)
    pts = rng.choice(np.concatenate([pts, -pts]), 3000).astype(np.float32)
    m_new, sym, q, _ = orc.ef_step(pts, np.zeros_like(pts), 0.0, E, M, bias)
    assert sym.dtype == np.uint16
    reps = sorted(set([Fraction(float(x)) for x in mag] + [-Fraction(float(x)) for x in mag]))
    for x, qq, s in zip(pts[:600], q[:600], sym[:600]):
        fx = Fraction(float(x))
        d = sorted((abs(fx - r), abs(r)) for r in reps)
        assert abs(Fraction(float(qq)) - fx) == d[0][0]                    # a nearest representative
        assert orc.value(int(s), E, M, bias) == float(qq)                   # the symbol names it
    v = pts + np.float32(0.0) * np.float32(0.0)                            # v = g + gamma m (so -0 becomes +0)
    assert np.array_equal((v - q).view(np.uint32), m_new.view(np.uint32))


def test_wide_round_trip_histogram_and_code():
    E, M, U = 5, 6, 2
    A = 1 << (1 + E + M)
    seg_len = [4096 + 70, 0, 3000]
    seg_book = [0, 1, 1]
    d = sum(seg_len)
    rng = np.random.default_rng(4)
    g = np.stack([syn.gennorm_numpy(rng, d, 0.9, 1e-3) for _ in range(U)])
    m = np.stack([syn.gennorm_numpy(rng, d, 1.0, 2e-4) for _ in range(U)])
    bias = np.full((U, 3), syn.bias_for_max(np.abs(g + np.float32(0.9) * m).max(), E), np.int32)
    enc = oround.encode_round(g, m, 0.9, E, M, seg_len, seg_book, bias)
    assert enc["sym"].dtype == np.uint16 and int(enc["sym"].max()) > 255 and enc["hist"].shape == (2, A)
    counts = np.zeros((2, A), np.uint64)
    off = 0
    for k, n in enumerate(seg_len):
        counts[seg_book[k]] += np.bincount(enc["sym"][:, off:off + n].ravel(), minlength=A).astype(np.uint64)
        off += n
    assert np.array_equal(counts, enc["hist"])
    for b in range(2):
        w = [int(x) for x in enc["hist"][b] if x]
        L = enc["lens"][b][enc["hist"][b] > 0].astype(int)
        assert sum(Fraction(1, 2 ** int(l)) for l in L) == 1                 # Kraft equality
        heap = list(w); heapq.heapify(heap); cost = 0
        while len(heap) > 1:
            a, c = heapq.heappop(heap), heapq.heappop(heap); cost += a + c; heapq.heappush(heap, a + c)
        assert int((enc["hist"][b].astype(object) * enc["lens"][b].astype(object)).sum()) == cost
    sym, avg = oround.ps_round(enc, E, M, seg_len, seg_book, bias)
    assert np.array_equal(sym, enc["sym"])                                   # h is invertible
    for i in (0, 1, 4095, 4096, d - 1):
        k = 0 if i < seg_len[0] else 2
        exact = sum(Fraction(orc.value(int(enc["sym"][u, i]), E, M, int(bias[u, k]))) for u in range(U)) / U
        assert abs(Fraction(float(avg[i])) - exact) <= abs(exact) * Fraction(1, 2 ** 23)


def test_wide_hand_stream():
    # two symbols above 255 with codes 0 and 1: the stream is their bit pattern, MSB first
    A = 1 << 10
    lens = np.zeros((1, A), np.uint8); codes = np.zeros((1, A), np.uint64)
    lens[0, 300] = 1; lens[0, 700] = 1; codes[0, 700] = 1
    sym = np.array([300, 700, 700, 300, 700], np.uint16)
    r = orc.pack(sym, [5], [0], lens, codes)
    assert r["rc"] == 0 and r["payload_bits"] == 5 and int(r["words"][0]) == 0b01101 << 27
    rc, back = orc.unpack(r["words"][:1], 5, [5], [0], lens, codes, r["chunk_offset"], r["sub_bits"])
    assert rc == 0 and np.array_equal(back, sym)


def test_wide_model_update_against_exact_rationals():
    # Algorithm 1 line 14 with 16-bit symbols: w - (eta / U) sum of representatives, against exact rational
    # arithmetic; eta = 0 leaves the model alone; U = 4, eta = 1, w = 0 is minus the (exact) average
    from fractions import Fraction
    E, M, U, d = 5, 6, 3, 200
    rng = np.random.default_rng(1801)
    nm = orc.num_magnitudes(E, M)
    sym = (rng.integers(0, nm, (U, d)) | (rng.integers(0, 2, (U, d)) << (E + M))).astype(np.uint16)
    sym[sym == (1 << (E + M))] = 0                       # no negative zero
    assert sym.max() > 255                               # beyond what a byte holds
    bias = rng.integers(18, 26, (U, 1)).astype(np.int32)
    w = rng.normal(0, 1e-2, d).astype(np.float32)
    eta = np.float32(0.37)
    got = orc.model_update(sym, [d], bias, E, M, eta, w)
    exact_round = np.empty(d, np.float32)
    for i in range(d):
        total = sum(Fraction(orc.value(int(sym[u, i]), E, M, int(bias[u, 0]))) for u in range(U))
        exact = Fraction(float(w[i])) - Fraction(float(eta)) * total / U
        exact_round[i] = np.float32(float(exact))
        assert abs(float(got[i]) - float(exact)) <= float(np.spacing(np.abs(exact_round[i]))), i
    assert np.mean(got == exact_round) > 0.99
    assert np.array_equal(orc.model_update(sym, [d], bias, E, M, 0.0, w), w)
    sym4 = np.concatenate([sym, sym[:1]])
    b4 = np.concatenate([bias, bias[:1]])
    avg = orc.aggregate(sym4, [d], b4, E, M)
    assert np.array_equal(orc.model_update(sym4, [d], b4, E, M, 1.0, np.zeros(d, np.float32)), -avg)


def test_wide_real_scale_special_cases_and_nearest_element():
    # the scaled conversion with 16-bit symbols: gain 1 is the plain step; a power-of-two gain is a shift of the
    # bias; for a general scale c every output is the nearest element of {c x} to the scaled input's pre-image,
    # checked in exact rationals on the representatives next to it; the average with inv_gain 1 is the plain one
    from fractions import Fraction
    import co3_synth as syn
    E, M, bias = 5, 5, 24
    rng = np.random.default_rng(1802)
    g = syn.gennorm_numpy(rng, 20_000, 0.9, 2e-3); m = syn.gennorm_numpy(rng, 20_000, 1.0, 5e-4)
    ref = orc.ef_step(g, m, 0.9, E, M, bias)
    got = orc.ef_step_gain(g, m, 0.9, E, M, bias, 1.0, 1.0)
    assert got[1].dtype == np.uint16 and got[1].max() > 255
    assert np.array_equal(ref[1], got[1]) and np.array_equal(ref[0].view(np.uint32), got[0].view(np.uint32))
    ref2 = orc.ef_step(g, m, 0.9, E, M, bias + 2)
    got2 = orc.ef_step_gain(g, m, 0.9, E, M, bias, 4.0, 0.25)
    assert np.array_equal(ref2[1], got2[1]) and np.array_equal(ref2[0].view(np.uint32), got2[0].view(np.uint32))
    assert np.array_equal(ref2[2].view(np.uint32), got2[2].view(np.uint32))
    # general scale: y = fl32(v s); the symbol's representative is the grid point nearest to y
    s_gain, c = np.float32(1.0 / 1.3), np.float32(1.3)
    mo, sym, q, _ = orc.ef_step_gain(g[:2000], np.zeros(2000, np.float32), 0.9, E, M, bias, s_gain, c)
    grid = orc.grid(E, M, bias)
    for i in range(2000):
        y = Fraction(float(np.float32(g[i] * s_gain)))
        k = int(sym[i]) & ((1 << (E + M)) - 1)
        mine = abs(abs(y) - Fraction(float(grid[k])))
        for kk in (k - 1, k + 1):
            if 0 <= kk < grid.size:
                assert mine <= abs(abs(y) - Fraction(float(grid[kk]))), i
        assert np.float32(q[i]) == np.float32(np.float32(orc.value(int(sym[i]), E, M, bias)) * c)
        assert np.float32(mo[i]) == np.float32(np.float32(g[i]) - np.float32(q[i]))
    two = np.stack([got[1][:500], ref2[1][:500]])
    b2 = np.array([[bias], [bias + 2]], np.int32)
    assert np.array_equal(orc.aggregate_gain(two, [500], b2, np.ones((2, 1), np.float32), E, M),
                          orc.aggregate(two, [500], b2, E, M))
