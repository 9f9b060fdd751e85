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
