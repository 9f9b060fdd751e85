"""Pins of the oracle's PS model update (eq. (aggregate hat), Algorithm 1 line 14): exact rational
arithmetic on the representatives, the cases where every step is exact, and consistency with the
averaging routine."""
from fractions import Fraction

import numpy as np

from oracle import co3_oracle as orc


def test_model_update_against_exact_rationals():
    E, M, U, d = 4, 3, 5, 400
    rng = np.random.default_rng(8)
    nm = orc.num_magnitudes(E, M)
    sym = (rng.integers(0, nm, (U, d)) | (rng.integers(0, 2, (U, d)) << (E + M))).astype(np.uint8)
    sym[sym == (1 << (E + M))] = 0                       # no negative zero
    bias = rng.integers(10, 18, (U, 1)).astype(np.int32)
    w = rng.normal(0, 1e-2, d).astype(np.float32)
    eta = np.float32(0.1)
    got = orc.model_update(sym, [d], bias, E, M, eta, w)
    for i in range(d):
        total = sum(Fraction(orc.value(int(sym[u, i]), E, M, int(bias[u, 0]))) for u in range(U))
        exact = Fraction(float(w[i])) - Fraction(float(eta)) * total / U
        # three fp64 roundings and one fp32 rounding away from the exact value: within one fp32 ulp,
        # and equal to the correctly rounded value unless the exact one sits next to a rounding boundary
        ref = np.float32(float(exact))
        assert abs(float(got[i]) - float(exact)) <= float(np.spacing(np.abs(ref))), i
    exact_round = np.array([np.float32(float(Fraction(float(w[i])) - Fraction(float(eta)) *
                            sum(Fraction(orc.value(int(sym[u, i]), E, M, int(bias[u, 0]))) for u in range(U)) / U))
                            for i in range(d)], np.float32)
    assert np.mean(got == exact_round) > 0.99


def test_model_update_exact_cases():
    E, M, d = 3, 2, 300
    rng = np.random.default_rng(9)
    nm = orc.num_magnitudes(E, M)
    sym = rng.integers(0, nm, (4, d)).astype(np.uint8)
    w = rng.normal(0, 1.0, d).astype(np.float32)
    # eta = 0: the model is unchanged
    assert np.array_equal(orc.model_update(sym, [d], [[5]] * 4, E, M, 0.0, w), w)
    # U = 4, eta = 1, w = 0: minus the average, which is exact (few mantissa bits, power-of-two 1/U)
    avg = orc.aggregate(sym, [d], np.full((4, 1), 5, np.int32), E, M)
    assert np.array_equal(orc.model_update(sym, [d], [[5]] * 4, E, M, 1.0, np.zeros(d, np.float32)), -avg)
    # U = 1, eta = 2 (a power of two), w = 0: minus twice the decoded value
    vals = np.array([orc.value(int(s), E, M, 5) for s in sym[0]])
    got = orc.model_update(sym[:1], [d], [[5]], E, M, 2.0, np.zeros(d, np.float32))
    assert np.array_equal(got, (-2.0 * vals).astype(np.float32))
    # layers with their own bias
    seg = [100, 0, 200]
    b = np.array([[5, 6, 7]] * 4, np.int32)
    got = orc.model_update(sym, seg, b, E, M, 1.0, np.zeros(d, np.float32))
    assert np.array_equal(got, -orc.aggregate(sym, seg, b, E, M))
