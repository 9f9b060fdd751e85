"""Pins for the GenNorm model weights (Sec. III eq. (gennorm), (kurtosis); Sec. IV-A (ii)) and
for the synthetic input generator that stands in for the paper's CNN gradients."""
import math

import numpy as np
import pytest
from scipy import special, stats

import co3_synth as syn
from oracle import co3_oracle as orc


@pytest.mark.parametrize("beta,alpha", [(1.0, 1e-3), (2.0, 3e-3), (0.7, 1e-4), (1.4, 1e-2)])
def test_generator_moments(beta, alpha):
    x = syn.gennorm_numpy(np.random.default_rng(1), 2_000_000, beta, alpha).astype(np.float64)
    var = alpha ** 2 * special.gamma(3 / beta) / special.gamma(1 / beta)            # eq. (kurtosis)
    kurt = special.gamma(5 / beta) * special.gamma(1 / beta) / special.gamma(3 / beta) ** 2
    assert abs(x.mean()) < 5 * math.sqrt(var / x.size)
    assert abs(x.var() / var - 1) < 0.02
    assert abs((x ** 4).mean() / x.var() ** 2 / kurt - 1) < 0.12


def test_cdf_special_cases_and_library():
    x = np.linspace(-0.02, 0.02, 401)
    F, S = orc.gennorm_cdf_pair(x, 1e-4, 2e-3, 1.0)                 # beta = 1: Laplace
    assert np.allclose(F, stats.laplace.cdf(x, 1e-4, 2e-3), rtol=1e-12, atol=0)
    F, S = orc.gennorm_cdf_pair(x, 0.0, 2e-3, 2.0)                  # beta = 2: Normal, sigma = alpha/sqrt 2
    assert np.allclose(F, stats.norm.cdf(x, 0, 2e-3 / math.sqrt(2)), rtol=1e-10, atol=1e-300)
    assert np.allclose(S, stats.norm.sf(x, 0, 2e-3 / math.sqrt(2)), rtol=1e-10, atol=1e-300)
    for beta in (0.6, 0.8, 1.3):
        F, S = orc.gennorm_cdf_pair(x, 0.0, 1e-3, beta)
        assert np.allclose(F, stats.gennorm.cdf(x, beta, 0, 1e-3), rtol=1e-9, atol=1e-300)
        assert np.allclose(S, stats.gennorm.sf(x, beta, 0, 1e-3), rtol=1e-9, atol=1e-300)


@pytest.mark.parametrize("E,M,beta", [(3, 0, 1.0), (4, 1, 0.8), (4, 3, 1.2), (5, 2, 0.7)])
def test_model_weights(E, M, beta):
    alpha = 1e-3
    x = syn.gennorm_numpy(np.random.default_rng(2), 3_000_000, beta, alpha)
    bias = syn.bias_for_max(np.abs(x).max(), E)
    w, p, syms = orc.gennorm_weights(E, M, bias, 0.0, alpha, beta)
    assert abs(p.sum() - 1) < 1e-12 and np.all(p >= 0)
    nm = orc.num_magnitudes(E, M)
    A = 1 << (1 + E + M)
    # weight > 0 exactly for the symbols Q_fp can emit
    can = np.zeros(A, bool); can[:nm] = True; can[(1 << (E + M)) + 1:(1 << (E + M)) + nm] = True
    assert np.array_equal(w > 0, can)
    # symmetric model: mirrored symbols have equal weight
    assert np.array_equal(w[1:nm], w[(1 << (E + M)) + 1:(1 << (E + M)) + nm])
    # empirical frequencies of quantized samples agree with the model cell masses
    _, code = orc.quantize_wide(x, E, M, bias)
    freq = np.bincount(code, minlength=A) / x.size
    pm = np.zeros(A); pm[syms] = p
    big = pm > 1e-4
    assert np.all(np.abs(freq[big] - pm[big]) < 6 * np.sqrt(pm[big] / x.size) + 1e-9)
    # the model book costs within a few percent of the empirical book on matching data
    le = orc.huffman_lengths(np.bincount(code, minlength=A).astype(np.uint64))
    lm = orc.huffman_lengths(w)
    cost_e = (freq * le).sum(); cost_m = (freq * lm).sum()
    assert cost_e <= cost_m < cost_e * 1.03 + 0.02
    assert lm.max() <= 64


def test_segments_and_bias_rule():
    s = syn.powerlaw_segments(138_357_544, 16)
    assert sum(s) == 138_357_544 and len(s) == 16 and all(x % 2 == 1 for x in s[1:]) and s[0] > s[-1]
    for E in (3, 4, 5):
        for mx in (1e-3, 0.75, 1.0, 1.9999, 2.0, 37.0):
            b = syn.bias_for_max(mx, E)
            g = orc.grid(E, 2, b)
            # top binade [2^emax, 2^(emax+1)) contains max|v|
            emax = (2 ** E - 2) - b
            assert 2.0 ** emax <= mx < 2.0 ** (emax + 1) and g[-1] == 1.75 * 2.0 ** emax
