"""Pins of the oracle's model-based exponent bias (oracle/co3_bias_model.py; eq. (exp bias) of
Sec. IV-A (i) with integer b): numerical quadrature of the defining integral with SciPy's GenNorm
density, Monte-Carlo with the oracle's quantizer (the paper's own route), closed forms of the
partial moments, and the exact power-of-two scaling law of the fp grid."""
import math

import numpy as np
import pytest
from scipy import integrate, stats

import co3_synth as syn
from oracle import co3_bias_model as bm
from oracle import co3_oracle as orc


def quad_sq_error(E, M, bias, mu, alpha, beta):
    """The definition, integrated cell by cell: sum_r int_cell (x - r)^2 f(x) dx."""
    mag = orc.grid(E, M, bias)
    reps = np.concatenate([-mag[:0:-1], mag])
    mids = 0.5 * (reps[:-1] + reps[1:])
    edges = np.concatenate([[-np.inf], mids, [np.inf]])
    pdf = stats.gennorm(beta, loc=mu, scale=alpha).pdf
    total = 0.0
    for r, a, b in zip(reps, edges[:-1], edges[1:]):
        val, _ = integrate.quad(lambda x: (x - r) ** 2 * pdf(x), a, b, epsabs=0, epsrel=1e-11, limit=200)
        total += val
    return total


def test_partial_moments_closed_forms():
    # whole line: mass 1, first moment 0, second moment = Var of eq. (kurtosis)
    for beta, alpha in [(0.7, 1e-3), (1.0, 2.0), (2.0, 0.3)]:
        assert abs(bm.interval_moment(0, -np.inf, np.inf, alpha, beta) - 1.0) < 1e-14
        assert abs(bm.interval_moment(1, -np.inf, np.inf, alpha, beta)) < 1e-18
        var = alpha ** 2 * math.gamma(3 / beta) / math.gamma(1 / beta)
        assert abs(bm.interval_moment(2, -np.inf, np.inf, alpha, beta) / var - 1.0) < 1e-13
    # Laplace(alpha): int_B^inf (x - B)^2 f = alpha^2 exp(-B / alpha) / 1 ... with f = exp(-x/alpha) / (2 alpha)
    alpha, B = 0.5, 1.7
    j0 = bm.interval_moment(0, B, np.inf, alpha, 1.0)
    j1 = bm.interval_moment(1, B, np.inf, alpha, 1.0)
    j2 = bm.interval_moment(2, B, np.inf, alpha, 1.0)
    assert abs((j2 - 2 * B * j1 + B * B * j0) / (alpha ** 2 * math.exp(-B / alpha)) - 1.0) < 1e-12
    # mirror symmetry and additivity over a split that straddles zero
    a, b = -0.4, 0.9
    for k in (0, 1, 2):
        whole = bm.interval_moment(k, a, b, 0.6, 1.3)
        parts = bm.interval_moment(k, a, 0.1, 0.6, 1.3) + bm.interval_moment(k, 0.1, b, 0.6, 1.3)
        assert abs(whole - parts) < 1e-15
        mirrored = bm.interval_moment(k, -b, -a, 0.6, 1.3)
        assert abs(whole - (-1) ** k * mirrored) < 1e-15


@pytest.mark.parametrize("E,M,beta,alpha,mu", [(2, 1, 1.0, 1.0, 0.0), (3, 0, 0.7, 1e-3, 0.0), (3, 2, 2.0, 0.05, 0.01),
                                              (4, 1, 1.4, 3e-3, -1e-3)])
def test_expected_error_equals_quadrature_of_the_definition(E, M, beta, alpha, mu):
    # biases around the one whose top binade holds the bulk of the distribution
    b0 = ((1 << E) - 2) - int(math.floor(math.log2(8 * alpha)))
    for bias in (b0 - 2, b0, b0 + 1, b0 + 3):
        closed = bm.expected_sq_error(E, M, bias, mu, alpha, beta)
        quad = quad_sq_error(E, M, bias, mu, alpha, beta)
        assert abs(closed / quad - 1.0) < 1e-8, (bias, closed, quad)


@pytest.mark.parametrize("E,M,beta", [(2, 1, 1.0), (4, 3, 0.8), (5, 2, 1.5)])
def test_expected_error_equals_monte_carlo_with_the_oracle_quantizer(E, M, beta):
    # the paper solves eq. (exp bias) by Monte-Carlo simulation: same quantity, sampled
    alpha = 1e-3
    rng = np.random.default_rng(17 + E)
    x = syn.gennorm_numpy(rng, 3_000_000, beta, alpha)
    b0 = ((1 << E) - 2) - int(math.floor(math.log2(np.abs(x).max())))
    for bias in (b0, b0 + 2, b0 + 4):
        err, _, _, _ = orc.ef_step(x, np.zeros_like(x), 0.0, E, M, bias, want_q=False)   # m' = v - Q(v)
        mc = float(np.mean(err.astype(np.float64) ** 2))
        model = bm.expected_sq_error(E, M, bias, 0.0, alpha, beta)
        assert abs(mc / model - 1.0) < 0.02, (bias, mc, model)


def test_power_of_two_scaling_law():
    # halving the scale and raising the bias by one halves every representative: error / 4, argmin + 1
    E, M, beta = 4, 3, 0.9
    for alpha in (1e-3, 0.37):
        for bias in (12, 17):
            e1 = bm.expected_sq_error(E, M, bias, 0.0, alpha, beta)
            e2 = bm.expected_sq_error(E, M, bias + 1, 0.0, alpha / 2, beta)
            assert abs(e1 / (4 * e2) - 1.0) < 1e-12
        b1, _ = bm.best_bias(E, M, 0.0, alpha, beta)
        b2, _ = bm.best_bias(E, M, 0.0, alpha / 2, beta)
        assert b2 == b1 + 1


@pytest.mark.parametrize("E,M,beta", [(2, 1, 1.0), (3, 2, 0.7), (4, 3, 1.0), (5, 2, 2.0)])
def test_best_bias_is_a_strict_local_and_global_minimum(E, M, beta):
    alpha = 2e-3
    b, e = bm.best_bias(E, M, 0.0, alpha, beta)
    errs = {c: bm.expected_sq_error(E, M, c, 0.0, alpha, beta) for c in bm.supported_biases(E)}
    lowest = min(errs.values())
    assert errs[b] == e and e <= lowest * (1 + bm.TIE)
    assert all(errs[c] > lowest * (1 + bm.TIE) for c in errs if c < b)     # the smallest bias of the plateau
    assert errs[b - 1] > e
    if E <= 4:                                                            # few binades: a strict minimum
        assert errs[b + 1] > e
    # the optimum trades clipping against resolution: with few binades its largest representative lies
    # between one and a few hundred standard deviations (with many, the plateau reaches further up)
    sigma = alpha * math.sqrt(math.gamma(3 / beta) / math.gamma(1 / beta))
    top = orc.grid(E, M, b)[-1]
    assert sigma < top
    if E <= 4:
        assert top < 1000 * sigma
    # no model: the IEEE bias
    assert bm.best_bias(E, M, 0.0, 0.0, 0.0) == ((1 << (E - 1)) - 1, 0.0)


def test_bias_table_shapes():
    par = np.array([[[0.0, 1e-3, 1.0, 6.0], [0.0, 0.0, 0.0, 0.0]], [[0.0, 4e-3, 1.0, 6.0], [0.0, 1e-2, 0.8, 9.0]]])
    bias, err = bm.bias_table(4, 3, par)
    assert bias.shape == (2, 2) and bias.dtype == np.int32
    assert bias[0, 1] == 7 and err[0, 1] == 0.0
    assert bias[0, 0] == bm.best_bias(4, 3, 0.0, 1e-3, 1.0)[0]
    assert bias[1, 0] == bias[0, 0] - 2       # scale four times larger
