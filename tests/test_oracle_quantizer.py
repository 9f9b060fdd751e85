"""Pins for the oracle's fp conversion Q_fp (Sec. IV-A (i), Sec. V-B of the paper).

None of these re-types the oracle's own search: the grid is rebuilt from the printed sets M
and E with exact rationals, the nearest value is found by a linear scan with exact rationals,
and three formats that coincide with IEEE half, bfloat16 and float8-e5m2 are checked against
NumPy / PyTorch casts.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import co3_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")

# formats of the five workloads plus the paper's fp4 [1,2,1] and fp8 [1,5,2]
FORMATS = [(3, 0), (4, 1), (4, 3), (3, 2), (5, 2), (2, 1), (2, 0), (2, 5), (7, 0)]


def paper_grid(E, M, bias):
    """X+ from the sets printed in Sec. V-B, as exact rationals, plus the zero/subnormal row."""
    b = (2 ** (E - 1) - 1) - bias
    c_scale = Fraction(2) ** b
    Mset = [1 + Fraction(a, 2 ** M) for a in range(2 ** M)]
    Eset = list(range(-(2 ** (E - 1) - 2), 2 ** (E - 1)))
    normal = sorted(c_scale * m * Fraction(2) ** e for e in Eset for m in Mset)
    sub = [c_scale * Fraction(a, 2 ** M) * Fraction(2) ** Eset[0] for a in range(2 ** M)]
    return sub + normal


@pytest.mark.parametrize("E,M", FORMATS)
def test_grid_matches_printed_sets(E, M):
    for bias in (0, 3, (2 ** (E - 1) - 1), 17):
        if not orc.format_ok(E, M, bias):
            continue
        g = orc.grid(E, M, bias)
        ref = paper_grid(E, M, bias)
        assert len(g) == len(ref) == 2 ** M * (2 ** E - 1)
        assert [Fraction(float(x)) for x in g] == ref
        assert all(g[i] < g[i + 1] for i in range(len(g) - 1))
        # number of symbols Q_fp can emit: every magnitude with both signs, zero once
        assert 2 * len(g) - 1 == 2 ** (M + 1) * (2 ** E - 1) - 1
        # boundary of eq. (quantizer boundary): B = c_scale (1 + 1/2 + ... + 2^-M) 2^max(E)
        b = (2 ** (E - 1) - 1) - bias
        B = Fraction(2) ** b * sum(Fraction(1, 2 ** i) for i in range(M + 1)) * Fraction(2) ** (2 ** (E - 1) - 1)
        assert Fraction(float(g[-1])) == B
        # value() agrees with the grid for both signs
        for k in (0, 1, len(g) // 2, len(g) - 1):
            assert orc.value(k, E, M, bias) == g[k]
            if k:
                assert orc.value((1 << (E + M)) | k, E, M, bias) == -g[k]


def test_grid_golden_fp4():
    rows = [l.split() for l in open(os.path.join(GOLD, "grid_fp4_121.txt")) if not l.startswith("#")]
    g = orc.grid(2, 1, 1)
    assert [(int(c), float(v)) for c, v in rows] == list(enumerate(g.tolist()))


def test_boundary_below_four_with_unit_L():
    # eq. (quantizer boundary): with c_scale = 2^-(2^(exp-1)-2) (L = 0) the boundary is < 4
    for E, M in FORMATS:
        b = -(2 ** (E - 1) - 2)
        bias = (2 ** (E - 1) - 1) - b
        g = orc.grid(E, M, bias)
        assert g[-1] == (2 - 2.0 ** -M) * 2 and g[-1] < 4
        assert g[2 ** M] == 1.0 * 2.0 ** b * 2.0 ** (-(2 ** (E - 1) - 2))


def nearest_exact(x: Fraction, grid, M):
    """Linear-scan argmin over the grid with exact arithmetic.  Tie: IEEE roundTiesToEven stated
    on the codes -- the even code for mant >= 1; for mant = 0 (one-digit significands, both odd)
    the larger magnitude, except that zero (significand 0, even) wins against the smallest value."""
    a = abs(x)
    best, bestd = [], None
    for k, m in enumerate(grid):
        dist = abs(a - m)
        if bestd is None or dist < bestd:
            best, bestd = [k], dist
        elif dist == bestd:
            best.append(k)
    if len(best) == 1:
        return best[0]
    lo, hi = best
    assert hi == lo + 1
    if M >= 1:
        return lo if lo % 2 == 0 else hi
    return lo if lo == 0 else hi


def probe_inputs(grid_f):
    """fp32 probes: grid points, midpoints, their fp32 neighbours, values beyond the top."""
    pts = []
    g32 = np.asarray(grid_f, dtype=np.float32)
    mids = (np.asarray(grid_f[:-1]) + np.asarray(grid_f[1:])) / 2
    for arr in (g32, mids.astype(np.float32)):
        pts += [arr, np.nextafter(arr, np.float32(np.inf)), np.nextafter(arr, np.float32(-np.inf))]
    top = np.float32(grid_f[-1])
    with np.errstate(over="ignore"):
        beyond = [top * np.float32(1.01), top * np.float32(2), top * np.float32(1e6)]
    pts.append(np.array(beyond + [ np.float32(1e-45), np.float32(3e-39),
                                  np.finfo(np.float32).max, np.finfo(np.float32).tiny], dtype=np.float32))
    with np.errstate(over="ignore"):
        x = np.concatenate(pts).astype(np.float32)
    x = x[np.isfinite(x)]
    return np.concatenate([x, -x])


@pytest.mark.parametrize("E,M", FORMATS)
def test_nearest_value_bruteforce(E, M):
    rng = np.random.default_rng(E * 100 + M)
    for bias in {(2 ** (E - 1) - 1), 10, 3 if E < 7 else 40}:
        if not orc.format_ok(E, M, bias):
            continue
        gf = orc.grid(E, M, bias)
        gq = [Fraction(float(v)) for v in gf]
        x = probe_inputs(gf)
        if len(x) > 1500:
            x = np.concatenate([x[:300], rng.choice(x, 1200, replace=False)])
        lo_e, hi_e = math.log2(gf[1]) - 3, math.log2(gf[-1]) + 2
        rnd = (2.0 ** rng.uniform(lo_e, hi_e, 400) * rng.choice([-1, 1], 400)).astype(np.float32)
        x = np.concatenate([x, rnd])
        q, code = orc.quantize_wide(x, E, M, bias)
        for xi, qi, ci in zip(x.tolist(), q.tolist(), code.tolist()):
            k = nearest_exact(Fraction(xi), gq, M)
            assert ci & ((1 << (E + M)) - 1) == k, (E, M, bias, xi)
            sign = ci >> (E + M)
            assert sign == (1 if (xi < 0 and k != 0) else 0)
            assert Fraction(qi) == (-gq[k] if sign else gq[k])


def test_m0_tie_rule_examples():
    # [1,3,0], bias 3: magnitudes 0, .25, .5, 1, 2, 4, 8.  One-digit significands: ties go to the
    # larger magnitude (IEEE 754-2019, 4.3.1), except 0.125 which lies between 0 and 0.25.
    q, c = orc.quantize_wide(np.array([0.125, 0.375, 0.75, 1.5, 3.0, 6.0, -6.0], np.float32), 3, 0, 3)
    assert q.tolist() == [0.0, 0.5, 1.0, 2.0, 4.0, 8.0, -8.0]
    assert c.tolist() == [0, 2, 3, 4, 5, 6, 8 | 6]


def ties_and_randoms(E, M, bias, rng, n=200000):
    """Random fp32 over the format's range plus every exact midpoint and its neighbours."""
    g = orc.grid(E, M, bias)
    lo_e, hi_e = math.log2(g[1]) - 4, math.log2(g[-1])
    x = (2.0 ** rng.uniform(lo_e, hi_e, n)).astype(np.float32)
    mids = ((g[:-1] + g[1:]) / 2).astype(np.float32)
    allx = np.concatenate([x, g.astype(np.float32), mids,
                           np.nextafter(mids, np.float32(np.inf)), np.nextafter(mids, np.float32(0))])
    return np.concatenate([allx, -allx])


def test_matches_ieee_half_cast():
    # [1,5,10] with bias 15 is IEEE binary16: NumPy's cast is a library reference below overflow
    x = ties_and_randoms(5, 10, 15, np.random.default_rng(1))
    x = x[np.abs(x) < 65520]
    q, _ = orc.quantize_wide(x, 5, 10, 15)
    ref = x.astype(np.float16).astype(np.float32)
    assert np.array_equal(q, ref)
    assert np.array_equal(np.signbit(q) & (q != 0), np.signbit(ref) & (ref != 0))


def test_matches_bfloat16_cast():
    import torch
    x = ties_and_randoms(8, 7, 127, np.random.default_rng(2), n=100000)
    x = x[np.isfinite(x) & (np.abs(x) < 3.38e38)]
    q, _ = orc.quantize_wide(x, 8, 7, 127)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(q, ref)


def test_matches_float8_e5m2_cast():
    # the paper's fp8, [1,5,2]; with bias 15 it is the e5m2 format of torch
    import torch
    x = ties_and_randoms(5, 2, 15, np.random.default_rng(3))
    x = x[np.abs(x) < 61440]
    q, _ = orc.quantize_wide(x, 5, 2, 15)
    ref = torch.from_numpy(x).to(torch.float8_e5m2).to(torch.float32).numpy()
    assert np.array_equal(q, ref)


@pytest.mark.parametrize("E,bias", [(3, 3), (5, 15), (4, 9)])
def test_m0_tie_rule_matches_the_e8m0_cast(E, bias):
    # mant = 0: every representative is a power of two, every midpoint a tie between two one-digit significands.
    # torch's float8_e8m0fnu (exponent-only, 2^-127 .. 2^127) is a library cast to the nearest power of two that
    # sends those ties to the larger magnitude, the rule of reading R3.  Compared on positive inputs inside the
    # format's normal range (e8m0 has neither sign nor zero).
    import torch
    if not hasattr(torch, "float8_e8m0fnu"):
        pytest.skip("this torch has no e8m0 cast")
    g = orc.grid(E, 0, bias)
    x = ties_and_randoms(E, 0, bias, np.random.default_rng(40 + E), n=50000)
    x = x[(x >= g[1]) & (x <= g[-1])]
    assert np.isin(((g[1:-1] + g[2:]) / 2).astype(np.float32), x).all()      # every tie between two powers of two is there
    q, _ = orc.quantize_wide(x, E, 0, bias)
    ref = torch.from_numpy(x).to(torch.float8_e8m0fnu).to(torch.float32).numpy()
    assert np.array_equal(q, ref)


def test_power_of_two_bias_is_a_pure_scaling():
    # c_scale = 2^b: changing the bias by k scales every representative by 2^-k (Sec. V-B)
    x = ties_and_randoms(5, 2, 15, np.random.default_rng(4), n=20000)
    q0, c0 = orc.quantize_wide(x, 5, 2, 15)
    for k in (-7, 5, 20):
        qk, ck = orc.quantize_wide(np.ldexp(x, -k).astype(np.float32), 5, 2, 15 + k)
        assert np.array_equal(ck, c0) and np.array_equal(qk, np.ldexp(q0, -k))


@pytest.mark.parametrize("E,M", [(3, 0), (4, 1), (4, 3), (3, 2), (5, 2)])
def test_error_bound_and_saturation(E, M):
    # proof of Lemma 1: inside +-B the error is at most half the local spacing, and at most
    # Delta/2 with Delta = c_scale 2^-mant 2^(2^(exp-1)-1); outside, the output is +-B
    bias = 2 ** (E - 1) + 2
    g = orc.grid(E, M, bias)
    B = g[-1]
    rng = np.random.default_rng(7)
    x = (rng.standard_normal(200000) * B / 2).astype(np.float32)
    q, code = orc.quantize_wide(x, E, M, bias)
    inside = np.abs(x) <= B
    b = (2 ** (E - 1) - 1) - bias
    Delta = 2.0 ** b * 2.0 ** -M * 2.0 ** (2 ** (E - 1) - 1)
    err = np.abs(x.astype(np.float64) - q)
    assert err[inside].max() <= Delta / 2
    ulp = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(np.abs(x), g[2 ** M]))) - M), g[1] if M else g[1])
    assert np.all(err[inside] <= ulp[inside] / 2 + 0)
    assert np.all(np.abs(q[~inside]) == B) and (~inside).sum() > 100
    assert np.all(np.sign(q[~inside]) == np.sign(x[~inside]))


def test_laplace_tail_closed_form():
    # proof of Lemma 1: with L = 0 and mant = 0 the boundary is B = 2, and for Laplace (beta = 1,
    # alpha = 1) E[(G - B)^2 ; G > B] = exp(-B) = 0.1353, the number behind the printed 0.15
    E, M = 3, 0
    b = -(2 ** (E - 1) - 2)
    bias = (2 ** (E - 1) - 1) - b
    rng = np.random.default_rng(11)
    x = rng.laplace(0.0, 1.0, 4_000_000).astype(np.float32)
    q, _ = orc.quantize_wide(x, E, M, bias)
    B = orc.grid(E, M, bias)[-1]
    assert B == 2.0
    tail = np.where(x > B, (x.astype(np.float64) - q) ** 2, 0.0).mean()
    assert abs(tail - math.exp(-B)) < 0.004
    assert tail <= 0.15


def test_nonfinite_and_zero():
    x = np.array([np.nan, np.inf, -np.inf, 0.0, -0.0, -1e-30], np.float32)
    q, c = orc.quantize_wide(x, 4, 3, 7)
    top = orc.grid(4, 3, 7)[-1]
    assert q[0] == 0 and c[0] == 0
    assert q[1] == top and q[2] == -top
    assert c[3] == 0 and c[4] == 0 and c[5] == 0 and not np.signbit(q[4]) and not np.signbit(q[5])


def test_format_limits():
    assert not orc.format_ok(1, 2, 0)            # the set E would be empty
    assert orc.format_ok(2, 1, 1)
    assert not orc.format_ok(4, 3, 200)          # subnormal step below 2^-149
    assert not orc.format_ok(4, 3, -120)         # top binade above 2^127
    assert orc.format_ok(4, 3, -113) and orc.format_ok(4, 3, 147)
