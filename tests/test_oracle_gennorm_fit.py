"""Pins of the oracle's GenNorm moment fit and pooled model weights (oracle/co3_gennorm_fit.py)
against what the paper and the mathematics fix: Sec. III eq. (kurtosis), the Laplace and Normal
special cases named there, closed-form three-point samples, SciPy's GenNorm moments, and
large seeded samples drawn by a generator that shares nothing with the fit."""
import math

import numpy as np
import pytest
from scipy import stats

import co3_synth as syn
from oracle import co3_gennorm_fit as fitm
from oracle import co3_oracle as orc


def test_kurtosis_closed_forms():
    # Sec. III: GenNorm subsumes Laplace (beta = 1, kurtosis 6) and Normal (beta = 2, kurtosis 3);
    # beta -> infinity is the uniform distribution (kurtosis 9/5)
    assert abs(fitm.kurtosis_of_beta(1.0) - 6.0) < 1e-12
    assert abs(fitm.kurtosis_of_beta(2.0) - 3.0) < 1e-12
    assert abs(fitm.kurtosis_of_beta(1e6) - 1.8) < 1e-5
    # Var / alpha^2: Laplace(alpha) has variance 2 alpha^2, Normal with alpha = sigma sqrt(2) has alpha^2 / 2
    assert abs(fitm.variance_factor(1.0) - 2.0) < 1e-12
    assert abs(fitm.variance_factor(2.0) - 0.5) < 1e-12


@pytest.mark.parametrize("beta", [0.3, 0.6, 0.8, 1.0, 1.4, 2.0, 3.5, 8.0])
def test_moments_match_scipy_gennorm(beta):
    var, exk = stats.gennorm.stats(beta, moments="vk")
    assert abs(fitm.variance_factor(beta) / float(var) - 1.0) < 1e-10
    assert abs(fitm.kurtosis_of_beta(beta) / (float(exk) + 3.0) - 1.0) < 1e-10


def test_kurtosis_falls_with_beta_and_inverse_round_trips():
    b = np.exp(np.linspace(np.log(fitm.BETA_MIN), np.log(fitm.BETA_MAX), 400))
    k = fitm.kurtosis_of_beta(b)
    assert np.all(np.diff(k) < 0)
    for beta in (0.11, 0.5, 0.9, 1.0, 1.7, 2.0, 5.0, 40.0):
        assert abs(fitm.beta_of_kurtosis(float(fitm.kurtosis_of_beta(beta))) / beta - 1.0) < 1e-10
    # outside the range: clamped
    assert fitm.beta_of_kurtosis(1.0) == fitm.BETA_MAX
    assert fitm.beta_of_kurtosis(1e9) == fitm.BETA_MIN
    assert fitm.beta_of_kurtosis(float("nan")) == fitm.BETA_MIN


def test_three_point_samples_closed_form():
    # {-1 (p), 0 (1 - 2p), +1 (p)}: mean 0, m2 = m4 = 2p, kurtosis 1 / (2p)
    mu, alpha, beta, kappa = fitm.fit([-1.0, 1.0] + [0.0] * 10)          # p = 1/12: kurtosis 6 -> Laplace
    assert mu == 0.0 and abs(kappa - 6.0) < 1e-12
    assert abs(beta - 1.0) < 1e-9 and abs(alpha - math.sqrt(1.0 / 12.0)) < 1e-9   # Var = 2 alpha^2 = 1/6
    mu, alpha, beta, kappa = fitm.fit([-1.0, 1.0] + [0.0] * 4)           # p = 1/6: kurtosis 3 -> Normal
    assert abs(kappa - 3.0) < 1e-12
    assert abs(beta - 2.0) < 1e-9 and abs(alpha - math.sqrt(2.0 / 3.0)) < 1e-9    # Var = alpha^2 / 2 = 1/3
    # shifted and scaled copy: mu moves, alpha scales, beta stays
    x = np.array([-1.0, 1.0] + [0.0] * 10) * 0.25 + 1000.0
    mu, alpha, beta, _ = fitm.fit(x)
    assert abs(mu - 1000.0) < 1e-9 and abs(beta - 1.0) < 1e-6 and abs(alpha - 0.25 * math.sqrt(1.0 / 12.0)) < 1e-9


def test_degenerate_samples():
    assert fitm.fit([]) == (0.0, 0.0, 0.0, 0.0)
    assert fitm.fit([3.0, 3.0, 3.0]) == (3.0, 0.0, 0.0, 0.0)
    # two-point sample: kurtosis 1, below every GenNorm: clamped at the uniform end
    assert fitm.fit([-1.0, 1.0])[2] == fitm.BETA_MAX


@pytest.mark.parametrize("beta,alpha", [(0.7, 1e-3), (1.0, 2e-3), (1.4, 5e-4), (2.0, 1e-2)])
def test_fit_recovers_generator_parameters(beta, alpha):
    # the workload generator (Gamma transform, co3_synth) shares nothing with the fit
    rng = np.random.default_rng(1234 + int(beta * 10))
    x = syn.gennorm_numpy(rng, 4_000_000, beta, alpha)
    mu, a, b, _ = fitm.fit(x)
    tol = 0.03 if beta < 1.0 else 0.015       # the fourth moment of a heavy tail converges slowly
    assert abs(mu) < 5e-3 * alpha
    assert abs(b / beta - 1.0) < tol
    assert abs(a / alpha - 1.0) < 2.5 * tol


def test_fit_on_library_laplace_and_normal_samples():
    rng = np.random.default_rng(77)
    mu, a, b, _ = fitm.fit(rng.laplace(0.5, 0.01, 4_000_000))
    assert abs(mu - 0.5) < 1e-4 and abs(b - 1.0) < 0.02 and abs(a / 0.01 - 1.0) < 0.03
    mu, a, b, _ = fitm.fit(rng.normal(-2.0, 0.1, 4_000_000))
    assert abs(mu + 2.0) < 1e-3 and abs(b - 2.0) < 0.03 and abs(a / (0.1 * math.sqrt(2.0)) - 1.0) < 0.02


def test_fit_round_uses_the_corrected_gradient():
    # v = fl32(g + fl32(gamma m)), per user and layer
    rng = np.random.default_rng(5)
    seg_len = [3000, 0, 5000]
    d = sum(seg_len)
    g = rng.laplace(0, 1e-3, (2, d)).astype(np.float32)
    m = rng.laplace(0, 5e-4, (2, d)).astype(np.float32)
    out = fitm.fit_round(g, m, 0.9, seg_len)
    v = g[1, 3000:] + np.float32(0.9) * m[1, 3000:]
    assert out.shape == (2, 3, 4)
    assert np.allclose(out[1, 2], fitm.fit(v), rtol=1e-12)
    assert tuple(out[0, 1]) == (0.0, 0.0, 0.0, 0.0)
    out0 = fitm.fit_round(g, m, 0.0, seg_len)       # gamma = 0: the memory plays no part
    assert np.allclose(out0[0, 0], fitm.fit(g[0, :3000]), rtol=1e-12)


def test_pooled_model_weights():
    E, M = 4, 3
    A = 256
    # one pair: the single-model weights
    par = np.array([[[0.0, 1e-3, 0.9, 0.0]]])
    w = fitm.pooled_model_weights(E, M, [[17]], par, [1000], [0], False)
    w1, _, _ = orc.gennorm_weights(E, M, 17, 0.0, 1e-3, 0.9)
    assert np.array_equal(w[0], w1)
    # two identical pairs: unchanged; table ids per user when per_user_books
    par2 = np.repeat(par, 2, axis=0)
    assert np.array_equal(fitm.pooled_model_weights(E, M, [[17], [17]], par2, [1000], [0], False)[0], w1)
    wp = fitm.pooled_model_weights(E, M, [[17], [17]], par2, [1000], [0], True)
    assert wp.shape == (2, A) and np.array_equal(wp[0], w1) and np.array_equal(wp[1], w1)
    # a mixture weighted by element counts, layers sharing one table
    par3 = np.array([[[0.0, 1e-3, 0.9, 0.0], [1e-4, 4e-3, 1.5, 0.0]]])
    wm = fitm.pooled_model_weights(E, M, [[17, 15]], par3, [1000, 3000], [0, 0], False)
    _, pa, sa = orc.gennorm_weights(E, M, 17, 0.0, 1e-3, 0.9)
    _, pb, sb = orc.gennorm_weights(E, M, 15, 1e-4, 4e-3, 1.5)
    mix = np.zeros(A); mix[sa] += 0.25 * pa; mix[sb] += 0.75 * pb
    assert abs(mix.sum() - 1.0) < 1e-12
    expect = np.maximum(1, np.floor(mix * 2.0 ** 40))
    prod = w1 > 0
    assert np.all(np.abs(wm[0][prod].astype(np.float64) - expect[prod]) <= 1.0 + 1e-9 * expect[prod])
    assert np.all(wm[0][~prod] == 0)
    # no contribution (alpha = 0, or an empty layer): every producible symbol gets weight 1
    w0 = fitm.pooled_model_weights(E, M, [[17, 17]], np.zeros((1, 2, 4)), [10, 0], [0, 1], False)
    assert np.array_equal(w0[0], prod.astype(np.uint64)) and np.array_equal(w0[1], prod.astype(np.uint64))
