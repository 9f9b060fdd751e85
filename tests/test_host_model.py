"""Host-side helpers of the library against the oracle (no GPU): GenNorm model weights.

Two independent incomplete-gamma codes may differ in the last place and flip a floor(), so the
comparison allows |dw| <= 1 + 1e-9 w; parity tests of the encoder feed integer weights."""
import numpy as np
import pytest

from oracle import co3_oracle as orc
from paper_2204_08211_amd import binding as B


@pytest.mark.parametrize("E,M,bias,mu,alpha,beta", [
    (3, 0, 12, 0.0, 1e-3, 1.0), (4, 1, 20, 0.0, 1e-3, 0.8), (4, 3, 18, 0.0, 3e-3, 0.6), (4, 3, 22, 0.0, 2e-4, 1.4),
    (3, 2, 15, 1e-4, 5e-4, 1.0), (5, 2, 30, 0.0, 1e-4, 0.7), (2, 1, 9, -2e-3, 1e-3, 2.0), (4, 3, 10, 0.0, 1e-3, 1.9),
])
def test_gennorm_weights_match_oracle(E, M, bias, mu, alpha, beta):
    w = B.co3_gennorm_weights(E, M, bias, mu, alpha, beta)
    ref, p, _ = orc.gennorm_weights(E, M, bias, mu, alpha, beta)
    assert np.array_equal(w > 0, ref > 0)
    diff = np.abs(w.astype(np.float64) - ref.astype(np.float64))
    assert np.all(diff <= 1 + 1e-9 * ref.astype(np.float64)), (diff.max(), ref[diff.argmax()])
    assert abs(w.sum() / 2.0 ** 40 - 1) < 1e-6 + w.size * 2.0 ** -40


def test_gennorm_weights_argument_checks():
    L = B.lib()
    import ctypes as C
    buf = (C.c_uint64 * 256)()
    assert L.co3_gennorm_weights(B.Format(4, 3), 18, 0.0, -1.0, 1.0, buf) == B.ERR_ARG
    assert L.co3_gennorm_weights(B.Format(4, 3), 18, 0.0, 1e-3, 0.0, buf) == B.ERR_ARG
    assert L.co3_gennorm_weights(B.Format(4, 3), 300, 0.0, 1e-3, 1.0, buf) == B.ERR_FORMAT
    assert L.co3_gennorm_weights(B.Format(4, 3), 18, 0.0, 1e-3, 1.0, None) == B.ERR_ARG


@pytest.mark.parametrize("E,M,mu,alpha,beta", [(2, 1, 0.0, 1.0, 1.0), (3, 2, 0.0, 2e-3, 0.7), (4, 3, 1e-4, 1e-3, 1.0),
                                              (4, 1, -2e-3, 5e-2, 1.6), (5, 2, 0.0, 1e-4, 2.0), (3, 0, 0.0, 3.0, 0.5)])
def test_library_bias_from_model_equals_the_oracle(E, M, mu, alpha, beta):
    # eq. (exp bias) with integer b: the library's own incomplete gamma against the oracle's SciPy-based one
    from oracle import co3_bias_model as bm
    b_lib, e_lib = B.co3_bias_from_model(E, M, mu, alpha, beta)
    b_ref, e_ref = bm.best_bias(E, M, mu, alpha, beta)
    assert b_lib == b_ref
    assert abs(e_lib / e_ref - 1.0) < 1e-9


def test_library_bias_from_model_without_a_model():
    assert B.co3_bias_from_model(4, 3, 0.0, 0.0, 0.0) == (7, 0.0)


# ---- eq. (exp bias) with real b on the host (co3_scale_from_model) -------------------------------------------

@pytest.mark.parametrize("E,M,beta,sigma", [(2, 1, 1.0, 1.0), (2, 1, 0.7, 3e-3), (3, 0, 1.4, 0.2), (3, 2, 0.8, 1e-3),
                                            (4, 3, 1.3, 5.0)])
def test_real_valued_scale_from_model_is_the_oracles_optimum(E, M, beta, sigma):
    import math
    from scipy import special
    from oracle import co3_bias_model as bm
    alpha = sigma * math.sqrt(math.exp(special.gammaln(1.0 / beta) - special.gammaln(3.0 / beta)))   # variance sigma^2
    bias, gain, inv_gain, err = B.co3_scale_from_model(E, M, 0.0, alpha, beta)
    ieee = (1 << (E - 1)) - 1
    reps = bm.signed_set(E, M, ieee)
    b_lib = (ieee - bias) + math.log2(inv_gain)
    # the library's triple, evaluated by the oracle, is the error the library reports ...
    assert abs(bm.scaled_sq_error(reps, b_lib, 0.0, alpha, beta) / err - 1.0) < 1e-6
    # ... and it is the oracle's optimum over real b, which is at least as good as the best integer
    lo = (ieee - bias) - 3.0
    b_opt, err_opt = bm.best_real_scale(reps, alpha, beta, lo=lo, hi=lo + 6.0)
    assert abs(err / err_opt - 1.0) < 1e-5, (b_lib, b_opt)
    b_int, err_int = B.co3_bias_from_model(E, M, 0.0, alpha, beta)
    assert err <= err_int * (1 + 1e-12)
    assert 2 ** -0.5 * (1 - 1e-6) <= inv_gain <= 2 ** 0.5 * (1 + 1e-6) and abs(gain * inv_gain - 1.0) < 1e-6
    # the split the oracle takes for the same b gives the same integer part
    ob, og, oi = bm.split_real_scale(E, b_lib)
    assert ob == bias and abs(float(oi) / inv_gain - 1.0) < 1e-6


def test_real_valued_scale_keeps_the_integer_result_where_nothing_is_gained():
    # [1,5,2] has a plateau of biases for a narrow source; no model at all gives the IEEE bias
    bias, gain, inv_gain, err = B.co3_scale_from_model(5, 2, 0.0, 1e-3, 1.0)
    b_int, err_int = B.co3_bias_from_model(5, 2, 0.0, 1e-3, 1.0)
    assert err <= err_int
    if (gain, inv_gain) == (1.0, 1.0):
        assert bias == b_int
    assert B.co3_scale_from_model(4, 3, 0.0, 0.0, 0.0) == (7, 1.0, 1.0, 0.0)
