"""Exponent bias from the model: the integer bias that minimises the expected squared error of the
fp conversion, eq. (exp bias) of Sec. IV-A (i),
    b_t = argmin_b E | c_sgn c_mant 2^(c_exp + b) - G_t |^2 ,
for G_t ~ GenNorm(mu, alpha, beta), with b restricted to the integers (power-of-two scale; the value
exponent of exponent field f is f - bias), and, for the comparison with the polynomial fits the paper prints
in Sec. IV-B, with b real (best_real_scale, monte_carlo_sq_error).  TEST INFRASTRUCTURE ONLY: only tests/,
__graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.

The paper solves eq. (exp bias) by Monte-Carlo simulation; for a GenNorm model the expectation has a
closed form in incomplete gamma functions, which is what this module evaluates (SciPy's gammainc /
gammaincc and gammaln are library steps):
  E (Q(X) - X)^2 = sum over representatives r of  int_cell(r) (x - r)^2 f(x) dx,
  int_0^t y^k f_Y(y) dy = alpha^k Gamma((k+1)/beta) / (2 Gamma(1/beta)) P((k+1)/beta, (t/alpha)^beta)
for the zero-location density f_Y (eq. (gennorm)) and t >= 0.
"""
import numpy as np
from scipy import special

from . import co3_oracle as orc

MAX_BIAS = 127           # smallest normal magnitude 2^(1 - bias) is a normal fp32
MAX_TOP_EXPONENT = 100   # (2^exp - 2) - bias <= 100: the range the library supports


def supported_biases(E):
    return list(range(((1 << E) - 2) - MAX_TOP_EXPONENT, MAX_BIAS + 1))


def _interval_moment(k, a, b, alpha, beta):
    """int_a^b y^k f_Y(y) dy for 0 <= a <= b <= inf (arrays), on the tail that keeps precision."""
    shape = (k + 1.0) / beta
    ck = np.exp(k * np.log(alpha) + special.gammaln(shape) - special.gammaln(1.0 / beta)) / 2.0
    with np.errstate(over="ignore"):
        ta = (a / alpha) ** beta
        tb = np.where(np.isinf(b), np.inf, (b / alpha) ** beta)
    pa = special.gammainc(shape, ta)
    lower = special.gammainc(shape, tb) - pa
    upper = special.gammaincc(shape, ta) - special.gammaincc(shape, tb)
    return ck * np.where(pa > 0.5, upper, lower)


def interval_moment(k, a, b, alpha, beta):
    """int_a^b y^k f_Y(y) dy for any a <= b (arrays, +-inf allowed), f_Y the zero-location GenNorm density."""
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    sign = -1.0 if k % 2 else 1.0
    pos = _interval_moment(k, np.maximum(a, 0.0), np.maximum(b, 0.0), alpha, beta)        # part in [0, inf)
    neg = sign * _interval_moment(k, np.maximum(-b, 0.0), np.maximum(-a, 0.0), alpha, beta)  # mirrored part
    return pos + neg


def expected_sq_error_of_set(reps, mu, alpha, beta):
    """E (Q(X) - X)^2 for X ~ GenNorm(mu, alpha, beta) and Q = nearest element of the ascending set reps;
    cells are bounded by the midpoints between neighbouring representatives."""
    reps = np.asarray(reps, np.float64)
    mids = 0.5 * (reps[:-1] + reps[1:])
    lo = np.concatenate([[-np.inf], mids]) - mu
    hi = np.concatenate([mids, [np.inf]]) - mu
    c = reps - mu
    j0 = interval_moment(0, lo, hi, alpha, beta)
    j1 = interval_moment(1, lo, hi, alpha, beta)
    j2 = interval_moment(2, lo, hi, alpha, beta)
    return float(np.sum(j2 - 2.0 * c * j1 + c * c * j0))


def signed_set(E, M, bias):
    """The representative set of Sec. V-B with this integer bias, both signs, ascending (reading R2: with zero
    and the subnormal row)."""
    mag = orc.grid(E, M, int(bias))
    return np.concatenate([-mag[:0:-1], mag])


def literal_set(E, M):
    """The set exactly as Sec. V-B prints it, c_scale = 1: c_mant = 1 + a / 2^mant, c_exp from -(2^(exp-1) - 2) to
    2^(exp-1) - 1, both signs; it has no zero and no subnormal row."""
    mag = sorted((1.0 + a / 2.0 ** M) * 2.0 ** e for e in range(-(2 ** (E - 1) - 2), 2 ** (E - 1)) for a in range(2 ** M))
    mag = np.array(mag)
    return np.concatenate([-mag[::-1], mag])


def scaled_sq_error(reps, log2_scale, mu, alpha, beta):
    """The objective of eq. (exp bias) for a real b = log2_scale: E |2^b r(X) - X|^2 with r the nearest element of
    2^b reps."""
    return expected_sq_error_of_set(np.asarray(reps, np.float64) * 2.0 ** log2_scale, mu, alpha, beta)


def best_real_scale(reps, alpha, beta, lo=-40.0, hi=40.0, step=1.0 / 16):
    """argmin over real b of eq. (exp bias) for a zero-mean GenNorm(alpha, beta): a scan of [lo, hi] in steps of
    `step` binades, then a golden-section search between the scan points next to the best one.  Returns
    (b, error)."""
    from scipy import optimize
    bs = np.arange(lo, hi + step / 2, step)
    errs = np.array([scaled_sq_error(reps, b, 0.0, alpha, beta) for b in bs])
    k = int(errs.argmin())
    a, c = bs[max(k - 1, 0)], bs[min(k + 1, bs.size - 1)]
    res = optimize.minimize_scalar(lambda b: scaled_sq_error(reps, b, 0.0, alpha, beta), bracket=(a, bs[k], c),
                                   method="golden", options=dict(xtol=1e-10)) if 0 < k < bs.size - 1 else None
    if res is not None and res.fun <= errs[k]:
        return float(res.x), float(res.fun)
    return float(bs[k]), float(errs[k])


def monte_carlo_sq_error(reps, log2_scale, x):
    """The paper's own route to eq. (exp bias): the mean of |2^b r(x) - x|^2 over samples x (fp64, nearest element
    by sorted search)."""
    r = np.asarray(reps, np.float64) * 2.0 ** log2_scale
    x = np.asarray(x, np.float64)
    k = np.clip(np.searchsorted(r, x), 1, r.size - 1)
    near = np.where(np.abs(x - r[k - 1]) <= np.abs(r[k] - x), r[k - 1], r[k])
    return float(np.mean((near - x) ** 2))


def expected_sq_error(E, M, bias, mu, alpha, beta):
    """E (Q_fp(X) - X)^2 for X ~ GenNorm(mu, alpha, beta) and the format's representative set with this
    bias (Sec. V-B); cells are bounded by the midpoints between neighbouring representatives."""
    return expected_sq_error_of_set(signed_set(E, M, bias), mu, alpha, beta)


def split_real_scale(E, log2_scale):
    """A real b of eq. (exp bias), taken relative to the set with the IEEE bias 2^(exp-1) - 1, as the library takes
    it (reading R16): the integer bias that carries the nearest power of two, and the fp32 pair (gain, inv_gain)
    for the rest, inv_gain = fl32(2^(b - round(b))) in [2^-1/2, 2^1/2] and gain = fl32(1 / inv_gain)."""
    k = int(np.round(log2_scale))
    inv_gain = np.float32(2.0 ** (log2_scale - k))
    return ((1 << (E - 1)) - 1) - k, np.float32(np.float32(1.0) / inv_gain), inv_gain


TIE = 1e-9   # errors within this relative distance of the minimum count as equal


def best_bias(E, M, mu, alpha, beta):
    """(bias, error of that bias): the supported integer bias with the smallest expected squared error.
    A format with many binades has a plateau of biases whose errors differ only by tail mass far
    below rounding; errors within TIE (relative) of the minimum count as equal and the smallest such
    bias, the one with the most headroom, is taken.  alpha <= 0 (no model) gives the IEEE bias
    2^(exp-1) - 1."""
    if not (alpha > 0.0 and beta > 0.0):
        return (1 << (E - 1)) - 1, 0.0
    cand = supported_biases(E)
    errs = [expected_sq_error(E, M, b, mu, alpha, beta) for b in cand]
    limit = min(errs) * (1.0 + TIE)
    for b, e in zip(cand, errs):
        if e <= limit:
            return b, e


def bias_table(E, M, params):
    """best_bias for an array of parameters [U][nseg][>=3] = (mu, alpha, beta, ...): (int32 [U][nseg],
    float64 [U][nseg])."""
    params = np.asarray(params, np.float64)
    U, nseg = params.shape[:2]
    bias = np.zeros((U, nseg), np.int32)
    err = np.zeros((U, nseg))
    for u in range(U):
        for k in range(nseg):
            bias[u, k], err[u, k] = best_bias(E, M, *params[u, k, :3])
    return bias, err
