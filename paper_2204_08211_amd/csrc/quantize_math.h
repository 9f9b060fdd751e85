// Device arithmetic of the fp conversion Q_fp (Sec. IV-A (i); representative set of Sec. V-B:
// +-2^b * c_mant * 2^c_exp, c_mant = 1 + a/2^mant, plus a zero/subnormal row at exponent
// field 0).  Exponent field f has value exponent f - bias.
//
// Rounding to the closest representative is done by one fp32 addition: adding
// C = 2^(e + 23 - mant), e = max(exponent of |v|, smallest normal exponent), makes the
// hardware round |v| to a multiple of the local spacing 2^(e - mant) with IEEE
// round-to-nearest-even on the significand counted in units of that spacing.
#pragma once

#include <stdint.h>

namespace co3 {

struct QConst {
    uint32_t max_bits;   // fp32 pattern of the largest magnitude B
    uint32_t min_fexp;   // fp32 exponent field of the smallest normal magnitude, 2^(1 - bias)
    uint32_t c_add;      // 23 - mant
    uint32_t mant;
};

__device__ __host__ inline QConst make_qconst(int E, int M, int bias)
{
    QConst c;
    const int emin = 1 - bias;
    const int emax = ((1 << E) - 2) - bias;
    c.max_bits = ((uint32_t)(emax + 127) << 23) | ((((uint32_t)1 << M) - 1u) << (23 - M));
    c.min_fexp = (uint32_t)(emin + 127);
    c.c_add = (uint32_t)(23 - M);
    c.mant = (uint32_t)M;
    return c;
}

// Host-checkable range of (format, bias): every magnitude is an fp32, normal magnitudes are
// normal fp32 numbers, and the rounding constant C stays finite.
__device__ __host__ inline bool format_supported(int E, int M, int bias)
{
    if (E < 2 || M < 0 || 1 + E + M > 8) return false;
    const int emin = 1 - bias;
    const int emax = ((1 << E) - 2) - bias;
    return emin >= -126 && emax <= 100;
}

// q = Q_fp(v).  sym = sign | magnitude code.  flags bit0: v is NaN/Inf, bit1: finite and clamped.
// NaN gives symbol 0; +-Inf and |v| > B give +-B.
__device__ inline void quantize(float v, const QConst &c, uint32_t sign_shift, uint32_t &sym, float &q,
                                uint32_t &flags)
{
    const uint32_t bits = __float_as_uint(v);
    const uint32_t a = bits & 0x7fffffffu;
    const uint32_t ac = a < c.max_bits ? a : c.max_bits;            // clamp |v| to B
    uint32_t fexp = ac >> 23;
    fexp = fexp > c.min_fexp ? fexp : c.min_fexp;                    // spacing never below the subnormal one
    const uint32_t cb = (fexp + c.c_add) << 23;                      // C = 2^(e + 23 - mant)
    const float C = __uint_as_float(cb);
    const float t = __fadd_rn(__uint_as_float(ac), C);               // rounds to the local spacing
    const uint32_t r = __float_as_uint(t) - cb;                      // significand in units of the spacing
    const float qa = __fsub_rn(t, C);                                // exact
    uint32_t code = ((fexp - c.min_fexp) << c.mant) + r;
    const bool nonfinite = a >= 0x7f800000u;
    const bool isnan_ = a > 0x7f800000u;
    flags = (nonfinite ? 1u : 0u) | ((a > c.max_bits && !nonfinite) ? 2u : 0u);
    code = isnan_ ? 0u : code;
    const uint32_t sgn = (code != 0u) ? (bits >> 31) : 0u;
    sym = (sgn << sign_shift) | code;
    q = __uint_as_float(__float_as_uint(qa) | (sgn << 31));
}

// fp32 pattern of the value of a symbol (exact: every representative is an fp32).
__device__ inline uint32_t symbol_value_bits(uint32_t sym, int E, int M, int bias)
{
    const uint32_t sign_shift = (uint32_t)(E + M);
    const uint32_t k = sym & (((uint32_t)1 << sign_shift) - 1u);
    const uint32_t s = (sym >> sign_shift) & 1u;
    const uint32_t f = k >> M;
    const uint32_t am = k & (((uint32_t)1 << M) - 1u);
    uint32_t bits;
    if (f != 0u) {
        bits = ((uint32_t)((int)f - bias + 127) << 23) | (am << (23 - M));
    } else if (am == 0u) {
        bits = 0u;
    } else {
        // subnormal row: am * 2^(1 - bias - M); normalise by hand so no fp mode is involved
        const int h = 31 - __builtin_clz(am);
        const int ex = h + 1 - bias - M;
        if (ex >= -126) bits = ((uint32_t)(ex + 127) << 23) | ((am << (23 - h)) & 0x7fffffu);
        else bits = am << (1 - bias - M + 149);
    }
    return bits | (s << 31);
}

}  // namespace co3
