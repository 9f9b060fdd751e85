"""Pins for the oracle's error-feedback step and PS average (Sec. IV-A (iii), Algorithm 1
lines 8, 10, 13-14; eq. (aggregate hat))."""
from fractions import Fraction

import numpy as np
import pytest

import co3_synth as syn
from oracle import co3_oracle as orc


def draw(n, beta, alpha, seed):
    return syn.gennorm_numpy(np.random.default_rng(seed), n, beta, alpha)


@pytest.mark.parametrize("E,M,gamma", [(3, 0, 0.9), (4, 1, 0.9), (4, 3, 0.5), (5, 2, 0.95), (2, 1, 0.7)])
def test_memory_is_the_quantization_error(E, M, gamma):
    # m_t = (g_t + gamma m_{t-1}) - ghat_t: "the memory term is equal to the quantization error"
    n = 50000
    m = np.zeros(n, np.float32)
    for it in range(4):
        g = draw(n, 0.9, 1e-3, 100 * E + it)
        v = (g + (np.float32(gamma) * m).astype(np.float32)).astype(np.float32)   # two fp32 roundings
        bias = syn.bias_for_max(np.abs(v).max(), E)
        m_new, sym, q, cnt = orc.ef_step(g, m, gamma, E, M, bias)
        q_ref, code_ref = orc.quantize_wide(v, E, M, bias)
        assert np.array_equal(q, q_ref) and np.array_equal(sym, code_ref.astype(np.uint8))
        top = orc.grid(E, M, bias)[-1]
        ok = np.abs(v) <= top
        # v - q is exactly representable in range: q + m' gives v back with no rounding
        assert np.array_equal((q + m_new).astype(np.float32)[ok], v[ok])
        assert np.array_equal(m_new.astype(np.float64), v.astype(np.float64) - q.astype(np.float64))
        assert cnt[0] == 0 and cnt[1] == (~ok).sum()
        # values of the symbols are the q's
        vals = np.array([orc.value(s, E, M, bias) for s in range(1 << (1 + E + M))])
        assert np.array_equal(vals[sym], q.astype(np.float64))
        m = m_new


def test_gamma_zero_means_no_error_feedback():
    # gamma = 0 "is essentially not using error feedback" (Sec. VI): output independent of m
    g = draw(20000, 1.0, 1e-3, 1)
    m1 = draw(20000, 1.0, 1e-2, 2)
    a = orc.ef_step(g, np.zeros_like(g), 0.0, 4, 3, 14)
    b = orc.ef_step(g, m1, 0.0, 4, 3, 14)
    assert np.array_equal(a[1], b[1]) and np.array_equal(a[0], b[0])
    q_direct, _ = orc.quantize_wide(g, 4, 3, 14)
    assert np.array_equal(a[2], q_direct)


def test_telescoping_sum_with_unit_decay():
    # gamma = 1: m_T = sum_t g_t - sum_t ghat_t (the identity behind w~_t - w^_t = eta m_t in
    # Sec. V-C).  Inputs on a coarse dyadic lattice so that every fp32 operation is exact.
    rng = np.random.default_rng(3)
    n, T = 4000, 6
    m = np.zeros(n, np.float32)
    sum_g = np.zeros(n, np.float64); sum_q = np.zeros(n, np.float64)
    for t in range(T):
        g = (rng.integers(-2000, 2000, n) * 2.0 ** -14).astype(np.float32)
        m, sym, q, cnt = orc.ef_step(g, m, 1.0, 4, 3, 10)
        assert cnt[1] == 0
        sum_g += g; sum_q += q
    assert np.array_equal(sum_g - sum_q, m.astype(np.float64))


def test_three_roundings_not_fused():
    # v = fl(g + fl(gamma m)): choose values where a fused multiply-add would differ
    gamma = np.float32(0.9)
    m = np.array([1.0000001, 3.3333333, 0.7777777], np.float32)
    g = np.array([-0.9, -3.0, -0.7], np.float32)
    t = (gamma * m).astype(np.float32)
    v_two = (g + t).astype(np.float32)
    v_fma = (g.astype(np.float64) + gamma.astype(np.float64) * m.astype(np.float64)).astype(np.float32)
    assert not np.array_equal(v_two, v_fma)
    # in range, m' + q reproduces v exactly, so it shows which v the oracle formed
    m_new, sym, q, _ = orc.ef_step(g, m, gamma, 5, 2, 15)
    assert np.array_equal((q.astype(np.float64) + m_new.astype(np.float64)), v_two.astype(np.float64))


def test_nonfinite_inputs_reset_memory():
    g = np.array([np.nan, np.inf, -np.inf, 1.0, 1e30], np.float32)
    m = np.zeros(5, np.float32)
    m_new, sym, q, cnt = orc.ef_step(g, m, 0.9, 4, 3, 7)
    top = orc.grid(4, 3, 7)[-1]
    assert m_new[:3].tolist() == [0, 0, 0] and sym[0] == 0
    assert q[1] == top and q[2] == -top and q[4] == top
    assert m_new[4] == np.float32(np.float32(1e30) - np.float32(top))
    assert cnt.tolist() == [3, 1]


def test_histogram_is_bincount():
    rng = np.random.default_rng(5)
    sym = rng.integers(0, 256, 100001).astype(np.uint8)
    h = orc.histogram(sym, 256)
    assert np.array_equal(h, np.bincount(sym, minlength=256).astype(np.uint64)) and h.sum() == sym.size
    h2 = orc.histogram(sym[:10], 256, h.copy())
    assert h2.sum() == sym.size + 10


def test_average_single_user_is_q_and_exact_cases():
    E, M = 4, 3
    g = draw(30000, 0.8, 1e-3, 8)
    bias = syn.bias_for_max(np.abs(g).max(), E)
    _, sym, q, _ = orc.ef_step(g, np.zeros_like(g), 0.9, E, M, bias)
    out = orc.aggregate(sym[None, :], [30000], [[bias]], E, M)
    assert np.array_equal(out, q)
    # U = 4 users sharing one bias, two layers with different biases: sums of <= 4 values that
    # span < 24 bits are exact, and 1/4 is a power of two: compare with exact rationals
    U, d, segs = 4, 5000, [1234, 3766]
    b = np.array([[bias, bias + 3]] * U, np.int32)
    rng = np.random.default_rng(9)
    nm = orc.num_magnitudes(E, M)
    syms = (rng.integers(0, nm, (U, d)) | (rng.integers(0, 2, (U, d)) << (E + M))).astype(np.uint8)
    syms[(syms & 0x7F) == 0] = 0
    out = orc.aggregate(syms, segs, b, E, M)
    for i in list(range(0, 40)) + list(range(1220, 1250)) + [d - 1]:
        k = 0 if i < segs[0] else 1
        exact = sum(Fraction(orc.value(int(syms[u, i]), E, M, int(b[u, k]))) for u in range(U)) / U
        assert Fraction(float(out[i])) == exact
    # U = 3: one rounding of the exact mean
    out3 = orc.aggregate(syms[:3], segs, b[:3], E, M)
    for i in range(0, 60):
        exact = sum(Fraction(orc.value(int(syms[u, i]), E, M, int(b[u, 0]))) for u in range(3)) / 3
        assert abs(Fraction(float(out3[i])) - exact) <= abs(exact) * Fraction(1, 2 ** 23)
