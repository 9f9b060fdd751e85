"""Pins of the oracle's stochastic fp conversion (Sec. II-B (ii): Q as a stochastic mapping;
non-subtractive dither): the published known-answer vectors of Philox4x32-10, the properties the
definition fixes (output is one of the two neighbours; representatives map to themselves; the
upper neighbour is taken with probability (|v| - lo) / (hi - lo), so the conversion is unbiased),
and the error-feedback identity."""
import numpy as np
import pytest

from oracle import co3_oracle as orc


def test_philox_known_answers():
    # known-answer vectors published with the generator (Salmon, Moraes, Dror, Shaw, SC'11; Random123)
    assert orc.philox4x32_10([0, 0, 0, 0], [0, 0]) == [0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8]
    assert orc.philox4x32_10([0xffffffff] * 4, [0xffffffff] * 2) == [0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd]
    assert orc.philox4x32_10([0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344], [0xa4093822, 0x299f31d0]) == \
        [0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1]


def neighbours(grid, a):
    hi = np.searchsorted(grid, a, side="right")
    hi = np.minimum(hi, grid.size - 1)
    lo = np.maximum(hi - 1, 0)
    return grid[lo], grid[hi]


@pytest.mark.parametrize("E,M,bias", [(2, 1, 1), (3, 0, 5), (4, 3, 14), (5, 2, 20), (5, 5, 22), (4, 7, 12)])
def test_output_is_a_neighbour_and_representatives_are_fixed_points(E, M, bias):
    rng = np.random.default_rng(E * 10 + M)
    grid = orc.grid(E, M, bias)
    n = 200_000
    v = (rng.laplace(0, grid[-1] / 6, n)).astype(np.float32)
    v[:2000] = rng.uniform(-grid[2], grid[2], 2000).astype(np.float32)      # the zero/subnormal row
    m_new, sym, q, cnt = orc.ef_step_sr(v, np.zeros_like(v), 0.0, E, M, bias, user=3, elem0=77, seed=12345)
    a = np.abs(v.astype(np.float64))
    inside = a < grid[-1]
    lo, hi = neighbours(grid, a)
    qa = np.abs(q.astype(np.float64))
    assert np.all((qa[inside] == lo[inside]) | (qa[inside] == hi[inside]))
    assert np.all(qa[~inside] == grid[-1]) and int(cnt[1]) == int(np.sum(a > grid[-1]))
    assert np.all(np.sign(q[qa > 0]) == np.sign(v[qa > 0]))
    # symbol and value agree; m' = fl32(v - q): unlike the closest representative, the far neighbour can
    # make the difference inexact, by at most half an ulp of it
    vals = np.array([orc.value(int(s), E, M, bias) for s in range(1 << (1 + E + M))])
    assert np.array_equal(vals[sym], q.astype(np.float64))
    exact = v.astype(np.float64) - q.astype(np.float64)
    assert np.array_equal(m_new[inside], exact.astype(np.float32)[inside])
    assert np.all(np.abs(m_new.astype(np.float64) - exact)[inside] <= np.abs(exact[inside]) * 2.0 ** -24)
    assert np.all(np.abs(exact[inside]) < (hi - lo)[inside] + 1e-300)
    # representatives: never moved
    reps = np.concatenate([grid, -grid[1:]]).astype(np.float32)
    _, _, q2, _ = orc.ef_step_sr(reps, np.zeros_like(reps), 0.0, E, M, bias, 0, 0, 999)
    assert np.array_equal(q2, reps)


@pytest.mark.parametrize("E,M,bias", [(3, 0, 5), (4, 3, 14), (4, 5, 14)])
def test_upper_neighbour_probability_and_unbiasedness(E, M, bias):
    grid = orc.grid(E, M, bias)
    n = 400_000
    for lo_i, frac in [(0, 0.25), (1, 0.7), (grid.size // 2, 0.1), (grid.size - 2, 0.5)]:
        lo, hi = grid[lo_i], grid[lo_i + 1]
        x = np.float32(lo + frac * (hi - lo))
        p = (float(x) - lo) / (hi - lo)
        v = np.full(n, x, np.float32)
        _, _, q, _ = orc.ef_step_sr(v, np.zeros_like(v), 0.0, E, M, bias, user=1, elem0=0, seed=lo_i + 1)
        up = float(np.mean(q.astype(np.float64) == hi))
        assert abs(up - p) < 4 * np.sqrt(p * (1 - p) / n) + 1e-6, (lo_i, up, p)
        assert abs(float(q.astype(np.float64).mean()) - float(x)) < 4 * (hi - lo) * np.sqrt(p * (1 - p) / n) + 1e-12
    # different users, seeds and positions draw different dithers; the same ones repeat
    v = np.full(4096, np.float32(grid[3] + 0.5 * (grid[4] - grid[3])), np.float32)
    z = np.zeros_like(v)
    base = orc.ef_step_sr(v, z, 0.0, E, M, bias, 0, 0, 5)[1]
    assert np.array_equal(base, orc.ef_step_sr(v, z, 0.0, E, M, bias, 0, 0, 5)[1])
    assert not np.array_equal(base, orc.ef_step_sr(v, z, 0.0, E, M, bias, 1, 0, 5)[1])
    assert not np.array_equal(base, orc.ef_step_sr(v, z, 0.0, E, M, bias, 0, 0, 6)[1])
    assert not np.array_equal(base, orc.ef_step_sr(v, z, 0.0, E, M, bias, 0, 4096, 5)[1])
    # element i of a vector gets the same random word whether the vector is processed whole or in slices
    whole = orc.ef_step_sr(np.tile(v, 2), np.tile(z, 2), 0.0, E, M, bias, 0, 0, 5)[1]
    assert np.array_equal(whole[4096:], orc.ef_step_sr(v, z, 0.0, E, M, bias, 0, 4096, 5)[1])


def test_non_finite_inputs_follow_the_deterministic_rule():
    E, M, bias = 4, 3, 14
    grid = orc.grid(E, M, bias)
    v = np.array([np.nan, np.inf, -np.inf, 1e30, -1e30], np.float32)
    m_new, sym, q, cnt = orc.ef_step_sr(v, np.zeros_like(v), 0.0, E, M, bias, 0, 0, 1)
    assert sym[0] == 0 and q[0] == 0 and m_new[0] == 0
    assert q[1] == np.float32(grid[-1]) and q[2] == -np.float32(grid[-1]) and m_new[1] == 0 and m_new[2] == 0
    assert q[3] == np.float32(grid[-1]) and q[4] == -np.float32(grid[-1])
    assert int(cnt[0]) == 3 and int(cnt[1]) == 2
