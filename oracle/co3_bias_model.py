"""Exponent bias from the model: the integer bias that minimises the expected squared error of the
fp conversion, eq. (exp bias) of Sec. IV-A (i),
    b_t = argmin_b E | c_sgn c_mant 2^(c_exp + b) - G_t |^2 ,
for G_t ~ GenNorm(mu, alpha, beta), with b restricted to the integers (power-of-two scale; the value
exponent of exponent field f is f - bias).  TEST INFRASTRUCTURE ONLY: only tests/,
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


def expected_sq_error(E, M, bias, mu, alpha, beta):
    """E (Q_fp(X) - X)^2 for X ~ GenNorm(mu, alpha, beta) and the format's representative set with this
    bias (Sec. V-B); cells are bounded by the midpoints between neighbouring representatives."""
    mag = orc.grid(E, M, int(bias))
    reps = np.concatenate([-mag[:0:-1], mag])
    mids = 0.5 * (reps[:-1] + reps[1:])
    lo = np.concatenate([[-np.inf], mids]) - mu
    hi = np.concatenate([mids, [np.inf]]) - mu
    c = reps - mu
    j0 = interval_moment(0, lo, hi, alpha, beta)
    j1 = interval_moment(1, lo, hi, alpha, beta)
    j2 = interval_moment(2, lo, hi, alpha, beta)
    return float(np.sum(j2 - 2.0 * c * j1 + c * c * j0))


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
