// Integer Huffman weights of the quantized symbols under the GenNorm gradient model
// (Sec. III, eq. (gennorm): f(x) = beta / (2 alpha Gamma(1/beta)) exp(-(|x - mu| / alpha)^beta);
// Sec. IV-A (ii): the code is designed under the GenNorm assumption).  Host-side helper, off
// the per-iteration path: the paper keeps the fitted parameters for several epochs (Sec. VI).
//
// The cell of a representative is the set of inputs Q_fp maps to it: bounded by the midpoints to
// its neighbours, the outermost cells reaching to infinity.  Its mass is a difference of the CDF
//   F(x) = 1/2 + 1/2 sgn(x - mu) P(1/beta, (|x - mu| / alpha)^beta)
// with P the regularised lower incomplete gamma function, evaluated on the tail that avoids
// cancellation.
#include <cmath>
#include <vector>

#include "co3_internal.h"
#include "quantize_math.h"

namespace {

// Regularised incomplete gamma functions P(a, x) and Q(a, x) = 1 - P(a, x): power series for
// x < a + 1, continued fraction (modified Lentz) otherwise.
void inc_gamma(double a, double x, double *P, double *Q)
{
    if (x <= 0.0) { *P = 0.0; *Q = 1.0; return; }
    if (std::isinf(x)) { *P = 1.0; *Q = 0.0; return; }
    const double lead = std::exp(a * std::log(x) - x - std::lgamma(a));
    if (x < a + 1.0) {
        double term = 1.0 / a, sum = term, ap = a;
        for (int n = 0; n < 2000; ++n) {
            ap += 1.0;
            term *= x / ap;
            sum += term;
            if (std::fabs(term) < std::fabs(sum) * 1e-17) break;
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
            if (std::fabs(d) < tiny) d = tiny;
            c = b + an / c;
            if (std::fabs(c) < tiny) c = tiny;
            d = 1.0 / d;
            const double del = d * c;
            h *= del;
            if (std::fabs(del - 1.0) < 1e-16) break;
        }
        *Q = lead * h;
        *P = 1.0 - *Q;
    }
}

// F(x) and 1 - F(x), each without cancellation
void gennorm_cdf(double x, double mu, double alpha, double beta, double *F, double *S)
{
    double P, Q;
    inc_gamma(1.0 / beta, std::pow(std::fabs(x - mu) / alpha, beta), &P, &Q);
    if (x >= mu) { *F = 0.5 + 0.5 * P; *S = 0.5 * Q; }
    else { *F = 0.5 * Q; *S = 0.5 + 0.5 * P; }
}

}  // namespace

extern "C" int co3_gennorm_weights(co3_format format, int32_t bias, double mu, double alpha, double beta,
                                   uint64_t *weights)
{
    if (!weights || !(alpha > 0.0) || !(beta > 0.0) || !std::isfinite(mu)) return CO3_ERR_ARG;
    const int E = format.exp_bits, M = format.mant_bits;
    if (!co3::format_supported(E, M, bias)) return CO3_ERR_FORMAT;
    const uint32_t A = 1u << (1 + E + M);
    const int nmag = ((1 << E) - 1) << M;
    // magnitudes by code: exponent field f, mantissa field a
    std::vector<double> mag(nmag);
    for (int k = 0; k < nmag; ++k) {
        const int f = k >> M, a = k & ((1 << M) - 1);
        mag[k] = f == 0 ? std::ldexp((double)a, 1 - bias - M) : std::ldexp((double)((1 << M) + a), f - bias - M);
    }
    // signed representatives in ascending order with their symbols
    std::vector<double> val;
    std::vector<uint32_t> symb;
    for (int k = nmag - 1; k >= 1; --k) { val.push_back(-mag[k]); symb.push_back((1u << (E + M)) | (uint32_t)k); }
    for (int k = 0; k < nmag; ++k) { val.push_back(mag[k]); symb.push_back((uint32_t)k); }
    const size_t n = val.size();
    std::vector<double> F(n + 1), S(n + 1);   // at the lower edge of cell i; index n: +infinity
    F[0] = 0.0; S[0] = 1.0; F[n] = 1.0; S[n] = 0.0;
    for (size_t i = 1; i < n; ++i) gennorm_cdf(0.5 * (val[i - 1] + val[i]), mu, alpha, beta, &F[i], &S[i]);
    for (uint32_t s = 0; s < A; ++s) weights[s] = 0;
    const double scale = std::ldexp(1.0, 40);
    for (size_t i = 0; i < n; ++i) {
        double p;
        if (F[i + 1] <= 0.5) p = F[i + 1] - F[i];
        else if (S[i] <= 0.5) p = S[i] - S[i + 1];
        else p = F[i + 1] - F[i];
        if (p < 0.0) p = 0.0;
        const double w = std::floor(p * scale);
        weights[symb[i]] = w < 1.0 ? 1ull : (uint64_t)w;
    }
    return CO3_OK;
}
