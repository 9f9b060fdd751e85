"""GenNorm parameters of a gradient layer by matching moments, and the model code weights of a
code table that several (user, layer) pairs share.  TEST INFRASTRUCTURE ONLY: only tests/,
__graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.

Sec. III, eq. (kurtosis) of the paper (arXiv 2204.08211) gives, for X ~ GenNorm(mu, alpha, beta),
    Mean(X) = mu,   Var(X) = alpha^2 Gamma(3/beta) / Gamma(1/beta),
    Kurt(X) = Gamma(5/beta) Gamma(1/beta) / Gamma(3/beta)^2.
The fit takes the sample mean, the sample central moments m2 and m4 (two passes, fp64), solves
Kurt(beta) = m4 / m2^2 for beta (the kurtosis falls strictly with beta) and sets alpha from the
variance.  The paper does not say how its "best fit" is computed; matching the three quantities it
prints is the reading taken here.  SciPy's log-gamma and root finder are library steps.
"""
import numpy as np
from scipy import optimize, special

from . import co3_oracle as orc

BETA_MIN = 0.1     # kurtosis about 3.3e4 ... and 1.8 (the uniform limit) at the other end
BETA_MAX = 64.0


def kurtosis_of_beta(beta):
    """Kurt(X) of eq. (kurtosis)."""
    b = np.asarray(beta, dtype=np.float64)
    return np.exp(special.gammaln(5.0 / b) + special.gammaln(1.0 / b) - 2.0 * special.gammaln(3.0 / b))


def variance_factor(beta):
    """Var(X) / alpha^2 of eq. (kurtosis)."""
    b = np.asarray(beta, dtype=np.float64)
    return np.exp(special.gammaln(3.0 / b) - special.gammaln(1.0 / b))


def sample_moments(v):
    """n, mean, central m2, central m4 of a sample, two passes in fp64."""
    x = np.asarray(v, dtype=np.float64).ravel()
    n = x.size
    if n == 0:
        return 0, 0.0, 0.0, 0.0
    mean = float(np.sum(x) / n)
    c = x - mean
    c2 = c * c
    return n, mean, float(np.sum(c2) / n), float(np.sum(c2 * c2) / n)


def beta_of_kurtosis(kappa):
    """The beta in [BETA_MIN, BETA_MAX] whose kurtosis is kappa (clamped to that range)."""
    if not np.isfinite(kappa):
        return BETA_MIN
    if kappa >= kurtosis_of_beta(BETA_MIN):
        return BETA_MIN
    if kappa <= kurtosis_of_beta(BETA_MAX):
        return BETA_MAX
    f = lambda lb: float(np.log(kurtosis_of_beta(np.exp(lb))) - np.log(kappa))
    lb = optimize.brentq(f, np.log(BETA_MIN), np.log(BETA_MAX), xtol=1e-15, rtol=1e-15, maxiter=500)
    return float(np.exp(lb))


def fit_from_moments(mean, m2, m4):
    """(mu, alpha, beta, kappa); a constant sample (m2 == 0) gives alpha = beta = 0."""
    if not (m2 > 0.0):
        return float(mean), 0.0, 0.0, 0.0
    kappa = m4 / (m2 * m2)
    beta = beta_of_kurtosis(kappa)
    alpha = float(np.sqrt(m2 / variance_factor(beta)))
    return float(mean), alpha, beta, float(kappa)


def fit(v):
    """GenNorm(mu, alpha, beta) matching mean, variance and kurtosis of the sample v."""
    n, mean, m2, m4 = sample_moments(v)
    return fit_from_moments(mean, m2, m4)


def fit_round(g, m, gamma, seg_len):
    """Parameters of v = fl32(g + fl32(gamma m)) (eq. (f_error_fb)) per user and layer:
    array [U][nseg][4] = (mu, alpha, beta, kappa)."""
    g = np.asarray(g, np.float32); m = np.asarray(m, np.float32)
    U = g.shape[0]
    out = np.zeros((U, len(seg_len), 4))
    off = 0
    for k, n in enumerate(seg_len):
        for u in range(U):
            v = (g[u, off:off + n] + (np.float32(gamma) * m[u, off:off + n]).astype(np.float32)).astype(np.float32)
            out[u, k] = fit(v)
        off += n
    return out


def pooled_model_weights(E, M, bias, params, seg_len, seg_book, per_user_books, scale_bits=40, gain=None):
    """Integer Huffman weights [nbooks][A] of the model code (Sec. IV-A (ii)) when table b serves the
    (user, layer) pairs mapped to it: the table's source is the mixture of the pairs' quantized
    GenNorm models weighted by their element counts; every symbol Q_fp can produce gets
    max(1, floor(p 2^scale_bits)).  Pairs with alpha == 0 or no elements contribute nothing; a table
    without contributions gets weight 1 on every producible symbol.  gain [U][nseg]: with a real-valued scale the
    conversion sees v gain, a GenNorm with location and scale multiplied by the gain."""
    params = np.asarray(params, np.float64)
    U, nseg = params.shape[:2]
    bias = np.broadcast_to(np.asarray(bias, np.int32), (U, nseg))
    A = 1 << (1 + E + M)
    bpu = max(seg_book) + 1
    nbooks = bpu * (U if per_user_books else 1)
    mass = np.zeros((nbooks, A))
    count = np.zeros(nbooks)
    emit = np.zeros((nbooks, A), bool)
    for u in range(U):
        for k in range(nseg):
            b = (u * bpu if per_user_books else 0) + seg_book[k]
            mu, alpha, beta = params[u, k, :3]
            if gain is not None:
                gn = float(np.asarray(gain, np.float32).reshape(U, nseg)[u, k])
                mu, alpha = mu * gn, alpha * gn
            _, p, syms = orc.gennorm_weights(E, M, int(bias[u, k]), 0.0, 1.0, 1.0, scale_bits)
            emit[b, syms] = True
            if seg_len[k] == 0 or not (alpha > 0.0 and beta > 0.0):
                continue
            _, p, syms = orc.gennorm_weights(E, M, int(bias[u, k]), mu, alpha, beta, scale_bits)
            mass[b, syms] += seg_len[k] * p
            count[b] += seg_len[k]
    w = np.zeros((nbooks, A), np.uint64)
    for b in range(nbooks):
        if count[b] > 0:
            p = mass[b] / count[b]
            w[b] = np.where(emit[b], np.maximum(1.0, np.floor(p * float(1 << scale_bits))), 0.0).astype(np.uint64)
        else:
            w[b] = emit[b].astype(np.uint64)
    return w
