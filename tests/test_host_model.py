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
