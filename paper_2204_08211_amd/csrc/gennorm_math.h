// GenNorm model arithmetic shared by the host helper and the device kernels of the library
// (Sec. III of the paper: eq. (gennorm) for the density, eq. (kurtosis) for variance and
// kurtosis; Sec. IV-A (ii): the Huffman code is designed under the GenNorm assumption).
//
//   f(x) = beta / (2 alpha Gamma(1/beta)) exp(-(|x - mu| / alpha)^beta)
//   F(x) = 1/2 + 1/2 sgn(x - mu) P(1/beta, (|x - mu| / alpha)^beta),  P the regularised lower
//          incomplete gamma function
//   Var  = alpha^2 Gamma(3/beta) / Gamma(1/beta),  Kurt = Gamma(5/beta) Gamma(1/beta) / Gamma(3/beta)^2
//
// The cell of a representative of Q_fp is the set of inputs mapped to it: bounded by the
// midpoints to its neighbours, the outermost cells reaching to infinity.
#pragma once

#include <math.h>
#include <stdint.h>

#if defined(__HIPCC__)
#define CO3_HD __host__ __device__
#else
#define CO3_HD
#endif

namespace co3 {

constexpr double kBetaMin = 0.1;    // range the moment fit searches; the kurtosis falls from
constexpr double kBetaMax = 64.0;   // about 3.3e4 to 1.8 (the uniform limit) over it

// Regularised incomplete gamma functions P(a, x) and Q(a, x) = 1 - P(a, x): power series for
// x < a + 1, continued fraction (modified Lentz) otherwise.
CO3_HD inline void inc_gamma(double a, double x, double *P, double *Q)
{
    if (x <= 0.0) { *P = 0.0; *Q = 1.0; return; }
    if (isinf(x)) { *P = 1.0; *Q = 0.0; return; }
    const double lead = exp(a * log(x) - x - lgamma(a));
    if (x < a + 1.0) {
        double term = 1.0 / a, sum = term, ap = a;
        for (int n = 0; n < 2000; ++n) {
            ap += 1.0;
            term *= x / ap;
            sum += term;
            if (fabs(term) < fabs(sum) * 1e-17) break;
        }
        *P = sum * lead;
        *Q = 1.0 - *P;
    } else {
        const double tiny = 1e-300;
        double b = x + 1.0 - a, c = 1.0 / tiny, d = 1.0 / b, h = d;
        for (int i = 1; i < 2000; ++i) {
            const double an = -(double)i * ((double)i - a);
            b += 2.0;
            d = an * d + b;
            if (fabs(d) < tiny) d = tiny;
            c = b + an / c;
            if (fabs(c) < tiny) c = tiny;
            d = 1.0 / d;
            const double del = d * c;
            h *= del;
            if (fabs(del - 1.0) < 4e-16) break;   // within an ulp of 1 (a tighter test can miss it for good)
        }
        *Q = lead * h;
        *P = 1.0 - *Q;
    }
}

// F(x) and 1 - F(x), each without cancellation; x may be +-infinity
CO3_HD inline void gennorm_cdf(double x, double mu, double alpha, double beta, double *F, double *S)
{
    double P, Q;
    inc_gamma(1.0 / beta, pow(fabs(x - mu) / alpha, beta), &P, &Q);
    if (x >= mu) { *F = 0.5 + 0.5 * P; *S = 0.5 * Q; }
    else { *F = 0.5 * Q; *S = 0.5 + 0.5 * P; }
}

// Probability of (lo, hi], taken on the tail that keeps precision.
CO3_HD inline double gennorm_mass(double lo, double hi, double mu, double alpha, double beta)
{
    double Flo, Slo, Fhi, Shi;
    gennorm_cdf(lo, mu, alpha, beta, &Flo, &Slo);
    gennorm_cdf(hi, mu, alpha, beta, &Fhi, &Shi);
    double p;
    if (Fhi <= 0.5) p = Fhi - Flo;
    else if (Slo <= 0.5) p = Slo - Shi;
    else p = Fhi - Flo;
    return p < 0.0 ? 0.0 : p;
}

// Magnitude of magnitude code k (exponent field k >> M, mantissa field below) for one bias.
CO3_HD inline double magnitude_of_code(int k, int M, int bias)
{
    const int f = k >> M, a = k & ((1 << M) - 1);
    return f == 0 ? ldexp((double)a, 1 - bias - M) : ldexp((double)((1 << M) + a), f - bias - M);
}

// Whether Q_fp can produce symbol s (the top exponent field and negative zero never occur), and
// the cell (lo, hi] of inputs it stands for.
CO3_HD inline bool symbol_cell(uint32_t s, int E, int M, int bias, double *lo, double *hi)
{
    const int nmag = ((1 << E) - 1) << M;
    const int k = (int)(s & ((1u << (E + M)) - 1u));
    const bool neg = ((s >> (E + M)) & 1u) != 0u;
    if (k >= nmag || (neg && k == 0) || (s >> (1 + E + M)) != 0u) return false;
    const double v = magnitude_of_code(k, M, bias);
    const double up = k == nmag - 1 ? INFINITY : 0.5 * (v + magnitude_of_code(k + 1, M, bias));
    if (k == 0) { *lo = -up; *hi = up; return true; }
    const double down = 0.5 * (v + magnitude_of_code(k - 1, M, bias));
    if (neg) { *lo = -up; *hi = -down; }
    else { *lo = down; *hi = up; }
    return true;
}

// int_a^b y^k f_Y(y) dy for the zero-location density f_Y and 0 <= a <= b <= infinity:
//   alpha^k Gamma((k+1)/beta) / (2 Gamma(1/beta)) [P((k+1)/beta, (b/alpha)^beta) - P(.., (a/alpha)^beta)],
// the difference taken on the tail that keeps precision.
CO3_HD inline double interval_moment_pos(int k, double a, double b, double alpha, double beta)
{
    if (!(b > a)) return 0.0;
    const double shape = ((double)k + 1.0) / beta;
    const double ck = 0.5 * exp((double)k * log(alpha) + lgamma(shape) - lgamma(1.0 / beta));
    double Pa, Qa, Pb, Qb;
    inc_gamma(shape, pow(a / alpha, beta), &Pa, &Qa);
    inc_gamma(shape, pow(b / alpha, beta), &Pb, &Qb);
    return ck * (Pa > 0.5 ? Qa - Qb : Pb - Pa);
}

// The same for any a <= b: the part on the negative axis is the mirrored integral with sign (-1)^k.
CO3_HD inline double interval_moment(int k, double a, double b, double alpha, double beta)
{
    const double pos = interval_moment_pos(k, a > 0.0 ? a : 0.0, b > 0.0 ? b : 0.0, alpha, beta);
    const double neg = interval_moment_pos(k, -b > 0.0 ? -b : 0.0, -a > 0.0 ? -a : 0.0, alpha, beta);
    return (k & 1) ? pos - neg : pos + neg;
}

// Share of symbol s in E (Q_fp(X) - X)^2 for X ~ GenNorm(mu, alpha, beta) and one exponent bias:
// the integral of (x - r)^2 f(x) over the cell of its representative r (0 if Q_fp cannot produce s).
CO3_HD inline double sq_error_of_symbol(uint32_t s, int E, int M, int bias, double mu, double alpha, double beta)
{
    double lo, hi;
    if (!symbol_cell(s, E, M, bias, &lo, &hi)) return 0.0;
    const int k = (int)(s & ((1u << (E + M)) - 1u));
    const double r = ((s >> (E + M)) & 1u) ? -magnitude_of_code(k, M, bias) : magnitude_of_code(k, M, bias);
    const double c = r - mu, a = lo - mu, b = hi - mu;
    const double j0 = interval_moment(0, a, b, alpha, beta);
    const double j1 = interval_moment(1, a, b, alpha, beta);
    const double j2 = interval_moment(2, a, b, alpha, beta);
    return j2 - 2.0 * c * j1 + c * c * j0;
}

// E (Q_fp(X) - X)^2: the objective of eq. (exp bias), Sec. IV-A (i), summed over the symbols.
CO3_HD inline double expected_sq_error(int E, int M, int bias, double mu, double alpha, double beta)
{
    const uint32_t A = 1u << (1 + E + M);
    double total = 0.0;
    for (uint32_t s = 0; s < A; ++s) total += sq_error_of_symbol(s, E, M, bias, mu, alpha, beta);
    return total;
}

// Candidate biases of the argmin: every bias the library supports for the format.
constexpr int kBiasMax = 127;
CO3_HD inline int bias_min_supported(int E) { return ((1 << E) - 2) - 100; }
constexpr double kBiasTie = 1e-9;  // errors within this relative distance of the minimum count as equal

// ln Kurt(beta) and Var / alpha^2 of eq. (kurtosis)
CO3_HD inline double log_kurtosis_of_beta(double b) { return lgamma(5.0 / b) + lgamma(1.0 / b) - 2.0 * lgamma(3.0 / b); }
CO3_HD inline double variance_factor(double b) { return exp(lgamma(3.0 / b) - lgamma(1.0 / b)); }

// The beta in [kBetaMin, kBetaMax] whose kurtosis is kappa (clamped to that range): bisection on
// ln beta; the kurtosis falls strictly with beta.
CO3_HD inline double beta_of_kurtosis(double kappa)
{
    if (!(kappa == kappa) || isinf(kappa)) return kBetaMin;
    const double lk = log(kappa);
    if (lk >= log_kurtosis_of_beta(kBetaMin)) return kBetaMin;
    if (lk <= log_kurtosis_of_beta(kBetaMax)) return kBetaMax;
    double lo = log(kBetaMin), hi = log(kBetaMax);
    for (int i = 0; i < 80; ++i) {
        const double mid = 0.5 * (lo + hi);
        if (log_kurtosis_of_beta(exp(mid)) > lk) lo = mid; else hi = mid;
    }
    return exp(0.5 * (lo + hi));
}

}  // namespace co3
