"""Pins of the oracle's real-valued scale (eq. (exp bias) of Sec. IV-A (i) with b in R; reading R16) and the
comparison with the polynomial fits of b_t that Sec. IV-B prints.

What pins the step (oracle/co3_oracle.c: co3o_ef_step_gain, co3o_aggregate_gain): gain 1 is the plain step; a
power-of-two gain equals a change of the integer bias (which fixes the direction of gain and inv_gain); the
outputs are the nearest elements of the scaled set c X found by brute force in exact arithmetic; the identity
m' = v - ghat in fp32.  What pins the argmin over real b (oracle/co3_bias_model.py): Monte-Carlo with samples of
the workload generator (the paper's route), the integer biases as special cases, local optimality.

The printed polynomials: read as a gain on the input (the set is scaled by 1 / b_t, which is what the division by
sigma suggests), the fp8 polynomial lies on the flat bottom of the objective over the whole range of beta the
paper plots; the fp4 polynomial agrees with the optimum only for beta between about 1.2 and 1.4 under that
reading, only near beta = 0.8 when b_t is read as the exponent offset of eq. (exp bias), and under no reading
over the whole range, with or without zero in the representative set.  Parity with them stays unpinned; the tests
below record exactly that.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import co3_synth as syn
from oracle import co3_bias_model as bm
from oracle import co3_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "bias_polynomials.txt")


def printed_polynomials():
    out = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        out[f[0]] = (int(f[1]), int(f[2]), [float(x) for x in f[3:]])
    return out


def unit_variance_alpha(beta):
    return math.sqrt(math.gamma(1.0 / beta) / math.gamma(3.0 / beta))   # Var = alpha^2 Gamma(3/beta) / Gamma(1/beta)


def test_gain_one_is_the_plain_step_and_a_power_of_two_gain_is_a_bias():
    E, M, bias = 4, 3, 16
    rng = np.random.default_rng(5)
    g = syn.gennorm_numpy(rng, 50_000, 0.9, 2e-3); m = syn.gennorm_numpy(rng, 50_000, 1.0, 5e-4)
    ref = orc.ef_step(g, m, 0.9, E, M, bias)
    got = orc.ef_step_gain(g, m, 0.9, E, M, bias, 1.0, 1.0)
    for a, b in zip(ref[:3], got[:3]):
        assert np.array_equal(a.view(np.uint32) if a.dtype == np.float32 else a, b.view(np.uint32) if b.dtype == np.float32 else b)
    # y = 4 v meets the set of `bias` exactly where v meets the set of bias + 2; ghat = value / 4 is that set's element
    ref2 = orc.ef_step(g, m, 0.9, E, M, bias + 2)
    got2 = orc.ef_step_gain(g, m, 0.9, E, M, bias, 4.0, 0.25)
    assert np.array_equal(ref2[1], got2[1]) and np.array_equal(ref2[0].view(np.uint32), got2[0].view(np.uint32))
    assert np.array_equal(ref2[2].view(np.uint32), got2[2].view(np.uint32))
    # the other direction (gain and inv_gain swapped) is a different quantizer
    swapped = orc.ef_step_gain(g, m, 0.9, E, M, bias, 0.25, 4.0)
    assert not np.array_equal(ref2[1], swapped[1])


@pytest.mark.parametrize("E,M,bias,c", [(2, 1, 1, 1.2345), (3, 2, 8, 0.77), (4, 3, 14, 1.4)])
def test_outputs_are_nearest_elements_of_the_scaled_set(E, M, bias, c):
    inv_gain = np.float32(c); gain = np.float32(np.float32(1.0) / inv_gain)
    mag = orc.grid(E, M, bias)
    top = float(mag[-1]) * c
    rng = np.random.default_rng(E * 10 + M)
    v = rng.uniform(-1.2 * top, 1.2 * top, 4000).astype(np.float32)
    m_new, sym, q, cnt = orc.ef_step_gain(v, np.zeros_like(v), 0.0, E, M, bias, gain, inv_gain)
    reps = [Fraction(float(np.float32(np.float32(x) * inv_gain))) for x in mag]     # fl32(value c), exactly
    reps = sorted(set([-r for r in reps] + reps))
    scaled = np.array([float(r) for r in reps])
    checked = 0
    for x, qq, mm in zip(v, q, m_new):
        fx = Fraction(float(x))
        d = sorted((abs(fx - r), r) for r in reps)
        # inputs within a relative 1e-5 of a cell boundary may fall either way (y = fl32(v gain) is rounded)
        if d[1][0] - d[0][0] <= Fraction(1, 100000) * abs(d[0][1] if d[0][1] else 1):
            continue
        assert Fraction(float(qq)) == d[0][1], (x, qq, float(d[0][1]))
        assert np.float32(x) - np.float32(qq) == mm                                  # m' = fl32(v - ghat)
        checked += 1
    assert checked > 3500 and set(np.unique(q)).issubset(set(scaled.astype(np.float32)))


def test_aggregate_with_scales():
    E, M, U, d = 3, 2, 3, 500
    rng = np.random.default_rng(9)
    bias = np.array([[6], [7], [5]], np.int32)
    inv_gain = np.array([[1.1], [0.8], [1.37]], np.float32)
    sym = np.stack([rng.integers(0, orc.num_magnitudes(E, M), d).astype(np.uint8) | (rng.integers(0, 2, d).astype(np.uint8) << 5)
                    for _ in range(U)])
    sym[sym == 32] = 0
    avg = orc.aggregate_gain(sym, [d], bias, inv_gain, E, M)
    for i in range(0, d, 37):
        vals = [Fraction(float(np.float32(np.float32(orc.value(int(sym[u, i]), E, M, int(bias[u, 0]))) * inv_gain[u, 0])))
                for u in range(U)]
        exact = sum(vals) / U
        assert abs(Fraction(float(avg[i])) - exact) <= abs(exact) * Fraction(1, 2 ** 23) + Fraction(1, 2 ** 140)
    one = orc.aggregate_gain(sym[:1], [d], bias[:1], inv_gain[:1], E, M)
    _, _, q, _ = orc.ef_step_gain(one, np.zeros_like(one), 0.0, E, M, int(bias[0, 0]), np.float32(1) / inv_gain[0, 0],
                                  inv_gain[0, 0])
    assert np.array_equal(one.view(np.uint32), q.view(np.uint32))     # a representative is a fixed point of the step


@pytest.mark.parametrize("E,M,beta", [(2, 1, 1.0), (3, 2, 0.7), (4, 3, 1.3)])
def test_real_scale_objective_equals_monte_carlo_and_beats_the_integers(E, M, beta):
    alpha = unit_variance_alpha(beta)
    reps = bm.signed_set(E, M, (1 << (E - 1)) - 1)
    b, err = bm.best_real_scale(reps, alpha, beta, lo=-12, hi=12)
    x = syn.gennorm_numpy(np.random.default_rng(3), 2_000_000, beta, alpha).astype(np.float64)
    assert abs(bm.monte_carlo_sq_error(reps, b, x) / err - 1.0) < 0.02
    assert abs(bm.monte_carlo_sq_error(reps, b + 0.7, x) / bm.scaled_sq_error(reps, b + 0.7, 0.0, alpha, beta) - 1.0) < 0.02
    # integer b are the special cases the library's bias covers: the real optimum is at least as good as the best
    # of them and not worse than its own neighbourhood
    ints = [bm.scaled_sq_error(reps, k, 0.0, alpha, beta) for k in range(-12, 13)]
    assert err <= min(ints) * (1 + 1e-12)
    assert abs(min(ints) / bm.best_bias(E, M, 0.0, alpha, beta)[1] - 1.0) < 1e-9
    for db in (-0.05, 0.05):
        assert bm.scaled_sq_error(reps, b + db, 0.0, alpha, beta) >= err
    # the split the library takes: integer bias + a factor within half a binade
    bias, gain, inv_gain = bm.split_real_scale(E, b)
    assert 2 ** -0.5 <= float(inv_gain) <= 2 ** 0.5 and abs(float(gain) * float(inv_gain) - 1.0) < 1e-6
    rebuilt = bm.signed_set(E, M, bias) * float(inv_gain)
    assert abs(bm.expected_sq_error_of_set(rebuilt, 0.0, alpha, beta) / err - 1.0) < 1e-5


@pytest.mark.parametrize("E,M,beta,shift", [(2, 1, 1.0, 0.3), (3, 2, 1.4, -0.8)])
def test_real_scale_objective_with_a_mean_equals_monte_carlo(E, M, beta, shift):
    # the closed form for a source whose mean is not zero (layers with a bias in their gradients), at two scales
    alpha = unit_variance_alpha(beta)
    reps = bm.signed_set(E, M, (1 << (E - 1)) - 1)
    x = syn.gennorm_numpy(np.random.default_rng(5), 2_000_000, beta, alpha).astype(np.float64) + shift
    for b in (-1.0, 0.37):
        assert abs(bm.monte_carlo_sq_error(reps, b, x) / bm.scaled_sq_error(reps, b, shift, alpha, beta) - 1.0) < 0.02
    # and moving the mean changes it
    assert abs(bm.scaled_sq_error(reps, 0.37, shift, alpha, beta) / bm.scaled_sq_error(reps, 0.37, 0.0, alpha, beta) - 1.0) > 0.02


def test_printed_fp8_polynomial_as_a_gain_lies_on_the_flat_bottom():
    E, M, coef = printed_polynomials()["fp8"]
    reps = bm.signed_set(E, M, (1 << (E - 1)) - 1)
    for beta in (0.4, 0.6, 0.8, 1.0, 1.2, 1.4, 1.6):
        alpha = unit_variance_alpha(beta)
        gain = sum(c * beta ** k for k, c in enumerate(coef))          # sigma = 1
        assert gain > 0
        err_poly = bm.scaled_sq_error(reps, -math.log2(gain), 0.0, alpha, beta)
        _, err_opt = bm.best_real_scale(reps, alpha, beta, lo=-20, hi=4, step=0.25)
        assert err_poly <= 1.015 * err_opt, (beta, err_poly, err_opt)


def test_printed_fp4_polynomial_matches_under_no_single_reading():
    E, M, coef = printed_polynomials()["fp4"]
    sets = {"with zero": bm.signed_set(E, M, (1 << (E - 1)) - 1), "as printed": bm.literal_set(E, M)}
    ratio = {}
    for name, reps in sets.items():
        for beta in (0.4, 0.8, 1.0, 1.2, 1.4):
            alpha = unit_variance_alpha(beta)
            p = sum(c * beta ** k for k, c in enumerate(coef))
            _, err_opt = bm.best_real_scale(reps, alpha, beta, lo=-6, hi=6)
            ratio[name, "gain", beta] = bm.scaled_sq_error(reps, -math.log2(p), 0.0, alpha, beta) / err_opt
            ratio[name, "scale", beta] = bm.scaled_sq_error(reps, math.log2(p), 0.0, alpha, beta) / err_opt
            ratio[name, "exponent", beta] = bm.scaled_sq_error(reps, p, 0.0, alpha, beta) / err_opt
    # where each reading does agree with the optimum
    assert ratio["with zero", "gain", 1.2] < 1.05 and ratio["with zero", "gain", 1.4] < 1.05
    assert ratio["with zero", "exponent", 0.8] < 1.02
    # and that none of them does over the range the paper plots
    for name in sets:
        for reading in ("gain", "scale", "exponent"):
            assert max(ratio[name, reading, beta] for beta in (0.4, 0.8, 1.0, 1.2, 1.4)) > 1.3, (name, reading)
