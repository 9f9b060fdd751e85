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
    if (E < 2 || M < 0 || 1 + E + M > 12) return false;   // up to 8 bits: byte symbols; 9 to 12: 16-bit symbols
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

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): counter-based generator, ten rounds.
struct Philox4 { uint32_t w[4]; };
__device__ __host__ inline Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                                 uint32_t k1)
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    Philox4 r;
    r.w[0] = c0; r.w[1] = c1; r.w[2] = c2; r.w[3] = c3;
    return r;
}

// The four random words of elements 4j .. 4j+3 of user u (element i takes word i mod 4).
__device__ inline Philox4 element_random_words(uint64_t elem, uint32_t user, uint64_t seed)
{
    const uint64_t j = elem >> 2;
    return philox4x32_10((uint32_t)j, (uint32_t)(j >> 32), user, 0u, (uint32_t)seed, (uint32_t)(seed >> 32));
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

// Stochastic fp conversion (Sec. II-B (ii): Q as a stochastic mapping, non-subtractive dither): v
// goes to the upper of its two neighbours with probability (|v| - lo) / (hi - lo).  A uniform
// integer dither is added to the position of |v| between them and the result truncated: in the
// normal range the position is the low 23 - mant bits of the fp32 pattern (the carry moves on to
// the next representative, across binades too); in the zero/subnormal row it is |v| in units of
// 2^(1 - bias - mant), truncated to 24 fractional bits.  rnd: this element's 32 random bits.
// Non-finite and clamped inputs as in quantize().
__device__ inline void quantize_stochastic(float v, const QConst &c, int E, int M, int bias, uint32_t sign_shift,
                                           uint32_t rnd, uint32_t &sym, float &q, uint32_t &flags)
{
    const uint32_t bits = __float_as_uint(v);
    const uint32_t a = bits & 0x7fffffffu;
    const uint32_t ac = a < c.max_bits ? a : c.max_bits;
    const bool nonfinite = a >= 0x7f800000u;
    flags = (nonfinite ? 1u : 0u) | ((a > c.max_bits && !nonfinite) ? 2u : 0u);
    uint32_t code, qbits;
    if (ac >= (c.min_fexp << 23)) {
        const uint32_t shift = c.c_add;                               // 23 - mant
        const uint32_t mask = (1u << shift) - 1u;
        qbits = (ac + (rnd >> (32u - shift))) & ~mask;                // never above max_bits
        code = (((qbits >> 23) - c.min_fexp + 1u) << c.mant) | ((qbits >> shift) & ((1u << c.mant) - 1u));
    } else {
        const uint32_t field = ac >> 23;
        const uint32_t mant24 = field ? ((ac & 0x7fffffu) | 0x800000u) : (ac & 0x7fffffu);
        const int sh = (field ? (int)field - 127 : -126) + M + bias;  // |v| = mant24 2^(e - 23); units of 2^(1-bias-M-24)
        const uint32_t xi = sh >= 0 ? mant24 << sh : (sh > -32 ? mant24 >> (-sh) : 0u);
        code = (xi + (rnd >> 8)) >> 24;                               // 0 .. 2^mant (the smallest normal)
        qbits = symbol_value_bits(code, E, M, bias);
    }
    code = (a > 0x7f800000u) ? 0u : code;                             // NaN
    const uint32_t sgn = (code != 0u) ? (bits >> 31) : 0u;
    sym = (sgn << sign_shift) | code;
    q = __uint_as_float((code != 0u ? qbits : 0u) | (sgn << 31));
}

}  // namespace co3
