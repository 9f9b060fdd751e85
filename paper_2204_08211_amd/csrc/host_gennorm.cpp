// Integer Huffman weights of the quantized symbols under the GenNorm gradient model
// (Sec. III, eq. (gennorm): f(x) = beta / (2 alpha Gamma(1/beta)) exp(-(|x - mu| / alpha)^beta);
// Sec. IV-A (ii): the code is designed under the GenNorm assumption).  Host-side helper, off
// the per-iteration path: the paper keeps the fitted parameters for several epochs (Sec. VI).
//
// The cell of a representative is the set of inputs Q_fp maps to it; its mass is a difference of
// the model's CDF (gennorm_math.h, shared with the device kernels that build the same weights
// from fitted parameters).
#include <cmath>
#include <vector>

#include "co3_internal.h"
#include "gennorm_math.h"
#include "quantize_math.h"

extern "C" int co3_gennorm_weights(co3_format format, int32_t bias, double mu, double alpha, double beta,
                                   uint64_t *weights)
{
    if (!weights || !(alpha > 0.0) || !(beta > 0.0) || !std::isfinite(mu)) return CO3_ERR_ARG;
    const int E = format.exp_bits, M = format.mant_bits;
    if (!co3::format_supported(E, M, bias)) return CO3_ERR_FORMAT;
    const uint32_t A = 1u << (1 + E + M);
    const double scale = std::ldexp(1.0, 40);
    for (uint32_t s = 0; s < A; ++s) {
        double lo, hi;
        if (!co3::symbol_cell(s, E, M, bias, &lo, &hi)) { weights[s] = 0; continue; }
        const double w = std::floor(co3::gennorm_mass(lo, hi, mu, alpha, beta) * scale);
        weights[s] = w < 1.0 ? 1ull : (uint64_t)w;
    }
    return CO3_OK;
}

// eq. (exp bias) with integer b for one parameter triple, on the host (same arithmetic as the
// device kernel k_model_bias).
extern "C" int co3_bias_from_model(co3_format format, double mu, double alpha, double beta, int32_t *bias,
                                   double *error)
{
    if (!bias || !std::isfinite(mu) || !(alpha >= 0.0) || !(beta >= 0.0)) return CO3_ERR_ARG;
    const int E = format.exp_bits, M = format.mant_bits;
    if (E < 2 || M < 0 || 1 + E + M > 12) return CO3_ERR_FORMAT;
    *bias = (1 << (E - 1)) - 1;
    if (error) *error = 0.0;
    if (!(alpha > 0.0) || !(beta > 0.0)) return CO3_OK;
    const int b0 = co3::bias_min_supported(E), n = co3::kBiasMax - b0 + 1;
    std::vector<double> err((size_t)n);
    double lowest = INFINITY;
    for (int i = 0; i < n; ++i) {
        err[(size_t)i] = co3::expected_sq_error(E, M, b0 + i, mu, alpha, beta);
        if (err[(size_t)i] < lowest) lowest = err[(size_t)i];
    }
    const double limit = lowest * (1.0 + co3::kBiasTie);
    for (int i = 0; i < n; ++i) {
        if (err[(size_t)i] <= limit) {
            *bias = b0 + i;
            if (error) *error = err[(size_t)i];
            break;
        }
    }
    return CO3_OK;
}

// eq. (exp bias) with real b for one parameter triple.  A scale c = 2^t on top of the integer bias turns the
// representative set into {c x}; the error of that set on GenNorm(mu, alpha, beta) equals c^2 times the error of
// the unscaled set on GenNorm(mu / c, alpha / c, beta), so the closed form of the integer case serves.
static double scaled_error(int E, int M, int bias, double t, double mu, double alpha, double beta)
{
    const double c = std::exp2(t);
    return c * c * co3::expected_sq_error(E, M, bias, mu / c, alpha / c, beta);
}

extern "C" int co3_scale_from_model(co3_format format, double mu, double alpha, double beta, int32_t *bias, float *gain,
                                    float *inv_gain, double *error)
{
    if (!bias || !gain || !inv_gain) return CO3_ERR_ARG;
    double err_int = 0.0;
    const int rc = co3_bias_from_model(format, mu, alpha, beta, bias, &err_int);
    if (rc != CO3_OK) return rc;
    *gain = 1.0f;
    *inv_gain = 1.0f;
    if (error) *error = err_int;
    if (!(alpha > 0.0) || !(beta > 0.0)) return CO3_OK;
    const int E = format.exp_bits, M = format.mant_bits;
    const int bmin = co3::bias_min_supported(E), bmax = co3::kBiasMax;
    // s = t - bias is the logarithm of the whole scale; bias = -round(s), t = s + bias in [-1/2, 1/2]
    auto split = [&](double s, int &b, double &t) {
        b = (int)std::lround(-s);
        if (b < bmin) b = bmin;
        if (b > bmax) b = bmax;
        t = s + (double)b;
    };
    auto f = [&](double s) {
        int b; double t;
        split(s, b, t);
        return scaled_error(E, M, b, t, mu, alpha, beta);
    };
    // scan one and a half binades to either side of the integer optimum in steps of 1/16, then a golden-section
    // search between the scan points next to the best one
    const double s0 = -(double)*bias;
    const int kHalf = 24;
    double best_s = s0, best_f = err_int;
    int best_k = 0;
    for (int k = -kHalf; k <= kHalf; ++k) {
        const double s = s0 + (double)k / 16.0, v = f(s);
        if (v < best_f) { best_f = v; best_s = s; best_k = k; }
    }
    if (best_k > -kHalf && best_k < kHalf) {
        const double r = 0.6180339887498949;
        double a = best_s - 1.0 / 16.0, b = best_s + 1.0 / 16.0;
        double x1 = b - r * (b - a), x2 = a + r * (b - a), f1 = f(x1), f2 = f(x2);
        for (int it = 0; it < 60; ++it) {
            if (f1 < f2) { b = x2; x2 = x1; f2 = f1; x1 = b - r * (b - a); f1 = f(x1); }
            else { a = x1; x1 = x2; f1 = f2; x2 = a + r * (b - a); f2 = f(x2); }
        }
        const double xm = 0.5 * (a + b), fm = f(xm);
        if (fm < best_f) { best_f = fm; best_s = xm; }
    }
    // a real scale is taken only where it helps: on the plateau of formats with many binades the integer bias stays
    if (!(best_f < err_int * (1.0 - co3::kBiasTie))) return CO3_OK;
    int b; double t;
    split(best_s, b, t);
    const float ig = (float)std::exp2(t);
    const float gn = 1.0f / ig;
    *bias = b;
    *gain = gn;
    *inv_gain = ig;
    if (error) *error = scaled_error(E, M, b, std::log2((double)ig), mu, alpha, beta);
    return CO3_OK;
}
