/*
 * CO3 gradient codec -- CPU ORACLE.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded implementation of what the CO3 per-iteration
 * path computes, written from the paper's definitions ("Communication-Efficient
 * Federated DNN Training: Convert, Compress, Correct", arXiv 2204.08211).  It
 * exists to check the GPU library and to be timed beside it.  Nothing in the
 * product may call it and it shares no code, table or header with the GPU path.
 *
 * Passages followed (section / equation / algorithm of the paper):
 *   - error correction with memory decay:  Sec. IV-A (iii), eq. (f_error_fb) and the
 *     memory recursion under it; Algorithm 1 lines 8 and 10.
 *   - fp conversion Q_fp:  Sec. IV-A (i); the representative set is the one of
 *     Sec. V-B "Quantization error bounding": c_sgn * c_scale * c_mant * 2^c_exp
 *     with c_mant in M, c_exp in E, c_scale = 2^b, input mapped to the closest.
 *   - element-wise Huffman coding h_Hf:  Sec. IV-A (ii); Sec. II-B (iii) (h is
 *     invertible, r = length of the binary string).
 *   - PS reconstruction and average:  Sec. II-B (iv), eq. (aggregate hat);
 *     Algorithm 1 lines 13-14.
 *
 * Where the paper is silent, ambiguous or at odds with itself the readings below
 * are taken:
 *   R1  exponent field f in [1, 2^exp - 2] <-> c_exp = f - (2^(exp-1) - 1); the
 *       integer parameter "bias" gives the value exponent f - bias, i.e. the
 *       paper's b is (2^(exp-1) - 1) - bias.
 *   R2  field f = 0 holds zero and IEEE-style subnormals (a / 2^mant) * 2^(1-bias);
 *       the top field 2^exp - 1 is never produced; a zero result has sign 0.
 *   R3  "closest": ties go to the neighbour whose significand, counted in units
 *       of the gap between the two neighbours, is even (IEEE 754 roundTiesToEven,
 *       including its one-digit-precision clause for mant = 0).
 *   R4  |v| above the largest magnitude B (and +-Inf) saturates to +-B.
 *       NaN gives symbol 0.  For NaN and +-Inf the new memory is 0.
 *   R5  v = fl32(g + fl32(gamma * m)), m' = fl32(v - q): three fp32 roundings.
 *   R6  Huffman: nodes ordered by (weight, key); a leaf's key is its symbol, an
 *       internal node's key is A + its creation order; the two smallest are merged.
 *       Lengths = depths; codes are the canonical ones (sorted by (length, symbol),
 *       first code 0, next = (prev + 1) << (length difference)).  One active
 *       symbol gets the 1-bit code "0".
 *   R7  container: bits are written MSB-first into 32-bit words; elements are cut
 *       into chunks of 4096 (restarting at every segment start), each chunk starts
 *       on a 32-bit boundary and consists of sub-chunks of 64 elements whose bit
 *       counts are stored beside the chunk's 64-bit bit offset.
 *   R8  average: sum over u = 0..U-1 in double, times 1.0/U, rounded to fp32.
 *       Model update w - (eta/U) sum: the same sum, times 1.0/U, times eta, subtracted
 *       from w in double, one rounding to fp32.
 *   R9  optional stochastic conversion (Sec. II-B (ii) allows Q to be a stochastic
 *       mapping): the upper neighbour with probability (|v| - lo) / (hi - lo), by an
 *       integer dither from Philox4x32-10; details at co3o_ef_step_sr.
 *
 *   R17 alphabets wider than one byte (1 + exp + mant up to 12 bits): the same steps with symbols
 *       stored in 16-bit words (functions with the suffix _w); nothing else changes.
 *
 * Parity pins (tests/, marker "not gpu"): grid against the sets M and E printed
 * in Sec. V-B; nearest-value brute force with exact rationals; IEEE half,
 * bfloat16 and float8-e5m2 casts of NumPy / PyTorch as special cases; error
 * bound Delta/2 and boundary B of Sec. V-B; Laplace tail closed form; Huffman
 * optimality by brute force, Kraft equality, dyadic / uniform / Fibonacci closed
 * forms, hand-worked tie-break cases; pack/unpack round trip and a hand-written
 * bitstream; error-feedback identity and telescoping sum; model update against
 * exact rationals; Philox known-answer vectors, neighbour / probability /
 * unbiasedness properties of the stochastic conversion.
 * Unpinned: the paper's own bits-per-element totals (Sec. VI) -- they are below
 * 1 bit/element, which an element-wise code cannot reach; "parity unpinned".
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fPIC -shared co3_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define CO3O_MAX_A 4096          /* symbols of the widest alphabet (1 + exp + mant = 12 bits) */
#define CO3O_CHUNK 4096u
#define CO3O_SUB 64u
#define CO3O_SUBS_PER_CHUNK (CO3O_CHUNK / CO3O_SUB)

enum {
    CO3O_OK = 0,
    CO3O_ERR_ARG = -1,
    CO3O_ERR_FORMAT = -2,
    CO3O_ERR_CAPACITY = -3,
    CO3O_ERR_CODELEN = -4,
    CO3O_ERR_CORRUPT = -5,
    CO3O_ERR_NOCODE = -7
};

/* Symbols are stored in bytes, or (suffix _w) in 16-bit words.               */
static inline uint32_t sym_get(const void *sym, int wide, uint64_t i)
{
    return wide ? ((const uint16_t *)sym)[i] : ((const uint8_t *)sym)[i];
}
static inline void sym_put(void *sym, int wide, uint64_t i, uint32_t s)
{
    if (wide) ((uint16_t *)sym)[i] = (uint16_t)s; else ((uint8_t *)sym)[i] = (uint8_t)s;
}

/* ------------------------------------------------------------------------- */
/* Representative set X (Sec. V-B).                                           */
/* ------------------------------------------------------------------------- */

/* Number of non-negative magnitudes of the format: one zero/subnormal row and
 * |E| = 2^exp - 2 normal rows, 2^mant values each.                           */
int co3o_num_magnitudes(int exp_bits, int mant_bits)
{
    return ((1 << exp_bits) - 1) << mant_bits;
}

/* Is [sgn,exp,mant] with this bias usable: every representative is an fp32.  */
int co3o_format_ok(int exp_bits, int mant_bits, int bias)
{
    if (exp_bits < 2 || exp_bits > 8 || mant_bits < 0 || mant_bits > 23) return 0;
    int fmax = (1 << exp_bits) - 2;
    if (1 - bias - mant_bits < -149) return 0; /* smallest subnormal step   */
    if (fmax - bias > 127) return 0;           /* largest binade            */
    return 1;
}

/* Magnitudes in increasing order; the index of a magnitude is its code
 * (exponent field << mant | mantissa field).  mag must hold
 * co3o_num_magnitudes() doubles.  Written as the paper writes X:
 * c_scale * c_mant * 2^c_exp over c_exp in E (ascending) and c_mant in M,
 * preceded by the zero/subnormal row of reading R2.                          */
int co3o_grid(int exp_bits, int mant_bits, int bias, double *mag)
{
    if (!co3o_format_ok(exp_bits, mant_bits, bias)) return CO3O_ERR_FORMAT;
    int nm = 1 << mant_bits;
    int ieee_bias = (1 << (exp_bits - 1)) - 1;
    int b = ieee_bias - bias;                         /* c_scale = 2^b       */
    int cexp_min = -((1 << (exp_bits - 1)) - 2);      /* min of the set E    */
    int cexp_max = (1 << (exp_bits - 1)) - 1;         /* max of the set E    */
    double c_scale = ldexp(1.0, b);
    int k = 0;
    for (int a = 0; a < nm; ++a)                      /* R2: zero, subnormals */
        mag[k++] = c_scale * ((double)a / nm) * ldexp(1.0, cexp_min);
    for (int c_exp = cexp_min; c_exp <= cexp_max; ++c_exp)
        for (int a = 0; a < nm; ++a) {
            double c_mant = 1.0 + (double)a / nm;     /* 1 + a_1/2 + ... */
            mag[k++] = c_scale * c_mant * ldexp(1.0, c_exp);
        }
    return k;
}

/* Closest representative of v (R3, R4).  Returns q; *code gets the magnitude
 * code with the sign bit placed above it; flags: bit0 = NaN/Inf, bit1 = finite
 * and clamped.                                                               */
static float quantize_one(const double *mag, int nmag, int sign_shift, float v,
                          uint32_t *code, int *flags)
{
    *flags = 0;
    if (isnan(v)) { *code = 0; *flags = 1; return 0.0f; }
    double a = fabs((double)v);
    int k;
    if (a >= mag[nmag - 1]) {
        k = nmag - 1;
        if (isinf(v)) *flags = 1;
        else if (a > mag[nmag - 1]) *flags = 2;
    } else {
        int lo = 0, hi = nmag - 1;            /* mag[lo] <= a < mag[hi]      */
        while (hi - lo > 1) {
            int mid = (lo + hi) / 2;
            if (mag[mid] <= a) lo = mid; else hi = mid;
        }
        double twice = 2.0 * a;               /* exact                       */
        double both = mag[lo] + mag[hi];      /* exact: neighbours           */
        if (twice < both) k = lo;
        else if (twice > both) k = hi;
        else {                                /* exact midpoint              */
            double gap = mag[hi] - mag[lo];
            double units = mag[lo] / gap;     /* significand of the lower one */
            k = (fmod(units, 2.0) == 0.0) ? lo : hi;
        }
    }
    uint32_t s = (signbit(v) && k != 0) ? 1u : 0u;
    *code = (s << sign_shift) | (uint32_t)k;
    double q = s ? -mag[k] : mag[k];
    return (float)q;                          /* exact by co3o_format_ok     */
}

/* Value of a symbol (sign | code).  Symbols that Q_fp never produces (top
 * exponent field, negative zero) are given the value NaN.                    */
double co3o_value(uint32_t sym, int exp_bits, int mant_bits, int bias)
{
    int nmag = co3o_num_magnitudes(exp_bits, mant_bits);
    uint32_t k = sym & ((1u << (exp_bits + mant_bits)) - 1u);
    uint32_t s = (sym >> (exp_bits + mant_bits)) & 1u;
    if ((int)k >= nmag || (s && k == 0)) return NAN;
    int f = (int)(k >> mant_bits);
    int a = (int)(k & ((1u << mant_bits) - 1u));
    double m = (f == 0) ? ldexp((double)a, 1 - bias - mant_bits)
                        : ldexp((double)((1 << mant_bits) + a), f - bias - mant_bits);
    return s ? -m : m;
}

/* Scalar fp conversion with wide codes, for formats beyond 8 bits (used to pin
 * the quantizer against library casts).                                      */
int co3o_quantize_wide(const float *v, uint64_t n, int exp_bits, int mant_bits,
                       int bias, float *q, uint32_t *code)
{
    int nmag = co3o_num_magnitudes(exp_bits, mant_bits);
    double *mag = (double *)malloc(sizeof(double) * (size_t)nmag);
    if (!mag) return CO3O_ERR_ARG;
    int rc = co3o_grid(exp_bits, mant_bits, bias, mag);
    if (rc < 0) { free(mag); return rc; }
    for (uint64_t i = 0; i < n; ++i) {
        int fl; uint32_t c;
        float qi = quantize_one(mag, nmag, exp_bits + mant_bits, v[i], &c, &fl);
        if (q) q[i] = qi;
        if (code) code[i] = c;
    }
    free(mag);
    return CO3O_OK;
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1, lines 8 and 10, for one user and one layer (one bias).        */
/*   v = g + gamma m ; q = Q_fp(v) ; m' = v - q   (R5)                        */
/* counters[0] += NaN/Inf inputs, counters[1] += finite clamped inputs.       */
/* m_out may alias m.  q_out may be NULL.                                     */
/* ------------------------------------------------------------------------- */
static int ef_step_any(const float *g, const float *m, uint64_t n, float gamma,
                       int exp_bits, int mant_bits, int bias,
                       float *m_out, void *sym, int wide, float *q_out, uint64_t *counters)
{
    if (1 + exp_bits + mant_bits > (wide ? 12 : 8)) return CO3O_ERR_FORMAT;
    int nmag = co3o_num_magnitudes(exp_bits, mant_bits);
    static double mag[CO3O_MAX_A];
    int rc = co3o_grid(exp_bits, mant_bits, bias, mag);
    if (rc < 0) return rc;
    for (uint64_t i = 0; i < n; ++i) {
        volatile float t = gamma * m[i];      /* fl32(gamma m)               */
        volatile float v = g[i] + t;          /* fl32(g + .)                 */
        int fl; uint32_t c;
        float q = quantize_one(mag, nmag, exp_bits + mant_bits, v, &c, &fl);
        volatile float err = v - q;           /* fl32(v - q)                 */
        if (fl & 1) err = 0.0f;               /* R4                          */
        if (counters) { counters[0] += (fl & 1); counters[1] += (fl >> 1) & 1; }
        sym_put(sym, wide, i, c);
        m_out[i] = err;
        if (q_out) q_out[i] = q;
    }
    return CO3O_OK;
}

int co3o_ef_step(const float *g, const float *m, uint64_t n, float gamma,
                 int exp_bits, int mant_bits, int bias,
                 float *m_out, uint8_t *sym, float *q_out, uint64_t *counters)
{
    return ef_step_any(g, m, n, gamma, exp_bits, mant_bits, bias, m_out, sym, 0, q_out, counters);
}

int co3o_ef_step_w(const float *g, const float *m, uint64_t n, float gamma,
                   int exp_bits, int mant_bits, int bias,
                   float *m_out, uint16_t *sym, float *q_out, uint64_t *counters)
{
    return ef_step_any(g, m, n, gamma, exp_bits, mant_bits, bias, m_out, sym, 1, q_out, counters);
}

/* ------------------------------------------------------------------------- */
/* Real-valued scale (eq. (exp bias) of Sec. IV-A (i) has b in R, i.e. a scale */
/* c_scale = 2^b that need not be a power of two).  Reading R16: the integer   */
/* bias carries the power-of-two part; on top of it the input is multiplied by */
/* a gain s before the conversion and the representative by c (the caller's    */
/* reciprocal of s) after it, all in fp32:                                     */
/*   y = fl32(v s),  sym = code of Q_fp(y),  ghat = fl32(value(sym) c),        */
/*   m' = fl32(v - ghat).                                                      */
/* The representative set is {c x : x in X}.  s = c = 1 is the plain step.     */
/* m' is no longer the exact difference (ghat is itself rounded).  Non-finite  */
/* y and clamping as R4, decided on y.                                         */
/* ------------------------------------------------------------------------- */
static int ef_step_gain_any(const float *g, const float *m, uint64_t n, float gamma,
                            int exp_bits, int mant_bits, int bias, float gain, float inv_gain,
                            float *m_out, void *sym, int wide, float *q_out, uint64_t *counters)
{
    if (1 + exp_bits + mant_bits > (wide ? 12 : 8)) return CO3O_ERR_FORMAT;
    int nmag = co3o_num_magnitudes(exp_bits, mant_bits);
    double mag[2048];
    int rc = co3o_grid(exp_bits, mant_bits, bias, mag);
    if (rc < 0) return rc;
    for (uint64_t i = 0; i < n; ++i) {
        volatile float t = gamma * m[i];
        volatile float v = g[i] + t;
        volatile float y = v * gain;          /* fl32(v s)                   */
        int fl; uint32_t c;
        volatile float qy = quantize_one(mag, nmag, exp_bits + mant_bits, y, &c, &fl);
        volatile float q = qy * inv_gain;     /* fl32(value c)               */
        volatile float err = v - q;
        if (fl & 1) err = 0.0f;
        if (counters) { counters[0] += (fl & 1); counters[1] += (fl >> 1) & 1; }
        sym_put(sym, wide, i, c);
        m_out[i] = err;
        if (q_out) q_out[i] = q;
    }
    return CO3O_OK;
}
int co3o_ef_step_gain(const float *g, const float *m, uint64_t n, float gamma,
                      int exp_bits, int mant_bits, int bias, float gain, float inv_gain,
                      float *m_out, uint8_t *sym, float *q_out, uint64_t *counters)
{
    return ef_step_gain_any(g, m, n, gamma, exp_bits, mant_bits, bias, gain, inv_gain, m_out, sym, 0, q_out, counters);
}
/* The same for alphabets of 9 to 12 bits (16-bit symbols). */
int co3o_ef_step_gain_w(const float *g, const float *m, uint64_t n, float gamma,
                        int exp_bits, int mant_bits, int bias, float gain, float inv_gain,
                        float *m_out, uint16_t *sym, float *q_out, uint64_t *counters)
{
    return ef_step_gain_any(g, m, n, gamma, exp_bits, mant_bits, bias, gain, inv_gain, m_out, sym, 1, q_out, counters);
}

/* ------------------------------------------------------------------------- */
/* Stochastic fp conversion (Sec. II-B (ii) allows Q to be a random mapping,   */
/* which is what non-subtractive dithering needs; the paper gives no          */
/* construction).  Reading: v goes to one of its two neighbours in X, the     */
/* upper one with probability (|v| - lo) / (hi - lo), decided by adding a     */
/* uniform integer dither to the position of |v| between them and truncating. */
/* The dither has as many bits as fp32 resolves between the neighbours        */
/* (23 - mant in the normal range) and 24 bits in the zero/subnormal row,     */
/* where the position is first truncated to 24 fractional bits.  Random bits: */
/* Philox4x32-10 (Salmon et al., SC'11), counter (i/4 low, i/4 high, user, 0) */
/* with i the element index within the user, key = the 64-bit seed; element i */
/* takes output word i mod 4.                                                 */
/* ------------------------------------------------------------------------- */
void co3o_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

static float quantize_one_sr(const double *mag, int nmag, int mant_bits, int sign_shift, float v,
                             uint32_t rnd, uint32_t *code, int *flags)
{
    *flags = 0;
    if (isnan(v)) { *code = 0; *flags = 1; return 0.0f; }
    double a = fabs((double)v);
    int k;
    if (a >= mag[nmag - 1]) {
        k = nmag - 1;
        if (isinf(v)) *flags = 1;
        else if (a > mag[nmag - 1]) *flags = 2;
    } else {
        int lo = 0, hi = nmag - 1;            /* mag[lo] <= a < mag[hi]      */
        while (hi - lo > 1) {
            int mid = (lo + hi) / 2;
            if (mag[mid] <= a) lo = mid; else hi = mid;
        }
        double pos = (a - mag[lo]) / (mag[hi] - mag[lo]);   /* in [0, 1), exact */
        int bits = (lo < (1 << mant_bits)) ? 24 : 23 - mant_bits;   /* zero/subnormal row : normal range */
        double scale = ldexp(1.0, bits);
        double units = floor(pos * scale);    /* exact already in the normal range */
        double dither = (double)(rnd >> (32 - bits));
        k = (units + dither >= scale) ? hi : lo;
    }
    uint32_t s = (signbit(v) && k != 0) ? 1u : 0u;
    *code = (s << sign_shift) | (uint32_t)k;
    double q = s ? -mag[k] : mag[k];
    return (float)q;
}

/* Algorithm 1 lines 8 and 10 with the stochastic conversion.  `user` and     */
/* `elem0` (index of g[0] within the user's vector) select the random words.  */
static int ef_step_sr_any(const float *g, const float *m, uint64_t n, float gamma,
                          int exp_bits, int mant_bits, int bias, uint32_t user, uint64_t elem0, uint64_t seed,
                          float *m_out, void *sym, int wide, float *q_out, uint64_t *counters)
{
    if (1 + exp_bits + mant_bits > (wide ? 12 : 8)) return CO3O_ERR_FORMAT;
    int nmag = co3o_num_magnitudes(exp_bits, mant_bits);
    double mag[2048];
    int rc = co3o_grid(exp_bits, mant_bits, bias, mag);
    if (rc < 0) return rc;
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    for (uint64_t i = 0; i < n; ++i) {
        uint64_t e = elem0 + i;
        uint32_t ctr[4] = {(uint32_t)(e >> 2), (uint32_t)((e >> 2) >> 32), user, 0u}, r[4];
        co3o_philox4x32_10(ctr, key, r);
        volatile float t = gamma * m[i];
        volatile float v = g[i] + t;
        int fl; uint32_t c;
        float q = quantize_one_sr(mag, nmag, mant_bits, exp_bits + mant_bits, v, r[e & 3u], &c, &fl);
        volatile float err = v - q;
        if (fl & 1) err = 0.0f;
        if (counters) { counters[0] += (fl & 1); counters[1] += (fl >> 1) & 1; }
        sym_put(sym, wide, i, c);
        m_out[i] = err;
        if (q_out) q_out[i] = q;
    }
    return CO3O_OK;
}
int co3o_ef_step_sr(const float *g, const float *m, uint64_t n, float gamma,
                    int exp_bits, int mant_bits, int bias, uint32_t user, uint64_t elem0, uint64_t seed,
                    float *m_out, uint8_t *sym, float *q_out, uint64_t *counters)
{
    return ef_step_sr_any(g, m, n, gamma, exp_bits, mant_bits, bias, user, elem0, seed, m_out, sym, 0, q_out, counters);
}
/* The same for alphabets of 9 to 12 bits (16-bit symbols). */
int co3o_ef_step_sr_w(const float *g, const float *m, uint64_t n, float gamma,
                      int exp_bits, int mant_bits, int bias, uint32_t user, uint64_t elem0, uint64_t seed,
                      float *m_out, uint16_t *sym, float *q_out, uint64_t *counters)
{
    return ef_step_sr_any(g, m, n, gamma, exp_bits, mant_bits, bias, user, elem0, seed, m_out, sym, 1, q_out, counters);
}

/* Symbol counts (the "distribution of the data source" that Huffman coding
 * requires, Sec. IV-A (ii)); adds into hist[0..A).                          */
void co3o_histogram(const uint8_t *sym, uint64_t n, uint64_t *hist)
{
    for (uint64_t i = 0; i < n; ++i) hist[sym[i]] += 1;
}
void co3o_histogram_w(const uint16_t *sym, uint64_t n, uint64_t *hist)
{
    for (uint64_t i = 0; i < n; ++i) hist[sym[i]] += 1;
}

/* ------------------------------------------------------------------------- */
/* Huffman code for integer weights (R6).                                     */
/* ------------------------------------------------------------------------- */
int co3o_huffman_lengths(const uint64_t *w, int A, uint8_t *len)
{
    if (A < 1 || A > CO3O_MAX_A) return CO3O_ERR_ARG;
    /* node store: leaves 0..A-1, internal nodes A.. in creation order       */
    static uint64_t weight[2 * CO3O_MAX_A]; static int parent[2 * CO3O_MAX_A]; static int alive[2 * CO3O_MAX_A];
    int n_active = 0, only = -1;
    uint64_t total = 0;
    for (int s = 0; s < A; ++s) {
        weight[s] = w[s]; parent[s] = -1; alive[s] = (w[s] > 0);
        len[s] = 0;
        if (w[s] > 0) {
            if (total + w[s] < total) return CO3O_ERR_ARG;   /* sum overflows */
            total += w[s]; ++n_active; only = s;
        }
    }
    if (n_active == 0) return 0;
    if (n_active == 1) { len[only] = 1; return 1; }
    int n_nodes = A;
    for (int step = 0; step < n_active - 1; ++step) {
        int pick[2];
        for (int r = 0; r < 2; ++r) {
            int best = -1;
            for (int i = 0; i < n_nodes; ++i) {         /* index order = key order */
                if (!alive[i]) continue;
                if (best < 0 || weight[i] < weight[best]) best = i;
            }
            alive[best] = 0;
            pick[r] = best;
        }
        weight[n_nodes] = weight[pick[0]] + weight[pick[1]];
        parent[n_nodes] = -1; alive[n_nodes] = 1;
        parent[pick[0]] = n_nodes; parent[pick[1]] = n_nodes;
        ++n_nodes;
    }
    int maxlen = 0;
    for (int s = 0; s < A; ++s) {
        if (w[s] == 0) continue;
        int depth = 0;
        for (int p = parent[s]; p >= 0; p = parent[p]) ++depth;
        if (depth > 64) return CO3O_ERR_CODELEN;
        len[s] = (uint8_t)depth;
        if (depth > maxlen) maxlen = depth;
    }
    return maxlen;
}

/* Canonical codes from lengths (R6): symbols with length 0 have no code.     */
int co3o_canonical_codes(const uint8_t *len, int A, uint64_t *code)
{
    static int order[CO3O_MAX_A]; int n = 0;
    if (A < 1 || A > CO3O_MAX_A) return CO3O_ERR_ARG;
    for (int s = 0; s < A; ++s) { code[s] = 0; if (len[s]) order[n++] = s; }
    for (int i = 1; i < n; ++i) {             /* insertion sort by (len, sym) */
        int s = order[i], j = i - 1;
        while (j >= 0 && (len[order[j]] > len[s] ||
                          (len[order[j]] == len[s] && order[j] > s))) {
            order[j + 1] = order[j]; --j;
        }
        order[j + 1] = s;
    }
    uint64_t c = 0;
    for (int i = 0; i < n; ++i) {
        if (i > 0) {
            int shift = len[order[i]] - len[order[i - 1]];
            c = c + 1;
            c = (shift >= 64) ? 0 : (c << shift);
        }
        code[order[i]] = c;
    }
    return CO3O_OK;
}

/* ------------------------------------------------------------------------- */
/* h_Hf: the binary string of one user (R7).                                  */
/* ------------------------------------------------------------------------- */
static void put_bit(uint32_t *words, uint64_t pos, int bit)
{
    if (bit) words[pos >> 5] |= (uint32_t)1 << (31 - (pos & 31));
}
static int get_bit(const uint32_t *words, uint64_t pos)
{
    return (int)((words[pos >> 5] >> (31 - (pos & 31))) & 1u);
}

/* Number of chunks of one user's vector for a list of layer lengths.         */
uint64_t co3o_num_chunks(int nseg, const uint64_t *seg_len)
{
    uint64_t n = 0;
    for (int k = 0; k < nseg; ++k) n += (seg_len[k] + CO3O_CHUNK - 1) / CO3O_CHUNK;
    return n;
}

/* Encode one user's symbols.  Layer k covers seg_len[k] consecutive elements
 * and uses code table seg_book[k] of len[.][A], code[.][A].
 * words[cap_words] is cleared and written; chunk_offset[nchunks+1] (bits),
 * sub_bits[nchunks*64] and *payload_bits (= r, the sum of codeword lengths)
 * are outputs.                                                               */
static int pack_any(const void *sym, int wide, int nseg, const uint64_t *seg_len,
                    const int32_t *seg_book, const uint8_t *len, const uint64_t *code,
                    int A, uint32_t *words, uint64_t cap_words,
                    uint64_t *chunk_offset, uint16_t *sub_bits, uint64_t *payload_bits)
{
    memset(words, 0, cap_words * sizeof(uint32_t));
    uint64_t pos = 0, payload = 0, chunk = 0, elem = 0;
    int rc = CO3O_OK;
    for (int k = 0; k < nseg; ++k) {
        const uint8_t *L = len + (size_t)seg_book[k] * A;
        const uint64_t *C = code + (size_t)seg_book[k] * A;
        for (uint64_t c0 = 0; c0 < seg_len[k]; c0 += CO3O_CHUNK, ++chunk) {
            pos = (pos + 31) & ~(uint64_t)31;           /* 32-bit boundary    */
            chunk_offset[chunk] = pos;
            uint64_t n_in_chunk = seg_len[k] - c0;
            if (n_in_chunk > CO3O_CHUNK) n_in_chunk = CO3O_CHUNK;
            for (uint32_t sc = 0; sc < CO3O_SUBS_PER_CHUNK; ++sc) {
                uint64_t start = pos;
                uint64_t j0 = (uint64_t)sc * CO3O_SUB;
                for (uint64_t j = j0; j < j0 + CO3O_SUB && j < n_in_chunk; ++j) {
                    uint32_t s = sym_get(sym, wide, elem + c0 + j);
                    if ((int)s >= A) { rc = CO3O_ERR_NOCODE; continue; }
                    int l = L[s];
                    if (l == 0) { rc = CO3O_ERR_NOCODE; continue; }
                    if (pos + (uint64_t)l > cap_words * 32) return CO3O_ERR_CAPACITY;
                    for (int b = l - 1; b >= 0; --b, ++pos)
                        put_bit(words, pos, (int)((C[s] >> b) & 1u));
                    payload += (uint64_t)l;
                }
                sub_bits[chunk * CO3O_SUBS_PER_CHUNK + sc] = (uint16_t)(pos - start);
            }
        }
        elem += seg_len[k];
    }
    pos = (pos + 31) & ~(uint64_t)31;
    chunk_offset[chunk] = pos;
    *payload_bits = payload;
    return rc;
}

int co3o_pack(const uint8_t *sym, int nseg, const uint64_t *seg_len,
              const int32_t *seg_book, const uint8_t *len, const uint64_t *code,
              int A, uint32_t *words, uint64_t cap_words,
              uint64_t *chunk_offset, uint16_t *sub_bits, uint64_t *payload_bits)
{
    return pack_any(sym, 0, nseg, seg_len, seg_book, len, code, A, words, cap_words, chunk_offset, sub_bits,
                    payload_bits);
}
int co3o_pack_w(const uint16_t *sym, int nseg, const uint64_t *seg_len,
                const int32_t *seg_book, const uint8_t *len, const uint64_t *code,
                int A, uint32_t *words, uint64_t cap_words,
                uint64_t *chunk_offset, uint16_t *sub_bits, uint64_t *payload_bits)
{
    return pack_any(sym, 1, nseg, seg_len, seg_book, len, code, A, words, cap_words, chunk_offset, sub_bits,
                    payload_bits);
}

/* Invert co3o_pack: walk the code tree bit by bit.  Reads nothing outside
 * words[0..n_words).                                                         */
static int unpack_any(const uint32_t *words, uint64_t n_words, int nseg,
                      const uint64_t *seg_len, const int32_t *seg_book,
                      const uint8_t *len, const uint64_t *code, int A,
                      const uint64_t *chunk_offset, const uint16_t *sub_bits,
                      void *sym, int wide)
{
    uint64_t chunk = 0, elem = 0;
    /* tree of the current book: child[node][bit]; >= 0 internal, -1 none,
     * leaves stored as -(2 + symbol)                                         */
    static int child[64 * CO3O_MAX_A + 2][2];
    if (A > CO3O_MAX_A) return CO3O_ERR_ARG;
    for (int k = 0; k < nseg; ++k) {
        const uint8_t *L = len + (size_t)seg_book[k] * A;
        const uint64_t *C = code + (size_t)seg_book[k] * A;
        int n_nodes = 1; child[0][0] = child[0][1] = -1;
        for (int s = 0; s < A; ++s) {
            if (!L[s]) continue;
            int node = 0;
            for (int b = L[s] - 1; b >= 0; --b) {
                int bit = (int)((C[s] >> b) & 1u);
                if (b == 0) {
                    if (child[node][bit] != -1) return CO3O_ERR_ARG; /* not prefix-free */
                    child[node][bit] = -(2 + s);
                } else {
                    if (child[node][bit] == -1) {
                        if (n_nodes >= 64 * CO3O_MAX_A + 2) return CO3O_ERR_ARG;
                        child[n_nodes][0] = child[n_nodes][1] = -1;
                        child[node][bit] = n_nodes++;
                    } else if (child[node][bit] < -1) return CO3O_ERR_ARG;
                    node = child[node][bit];
                }
            }
        }
        for (uint64_t c0 = 0; c0 < seg_len[k]; c0 += CO3O_CHUNK, ++chunk) {
            uint64_t pos = chunk_offset[chunk];
            if (pos & 31) return CO3O_ERR_CORRUPT;
            uint64_t n_in_chunk = seg_len[k] - c0;
            if (n_in_chunk > CO3O_CHUNK) n_in_chunk = CO3O_CHUNK;
            for (uint32_t sc = 0; sc < CO3O_SUBS_PER_CHUNK; ++sc) {
                uint64_t end = pos + sub_bits[chunk * CO3O_SUBS_PER_CHUNK + sc];
                if (end > n_words * 32) return CO3O_ERR_CORRUPT;
                uint64_t j0 = (uint64_t)sc * CO3O_SUB;
                for (uint64_t j = j0; j < j0 + CO3O_SUB && j < n_in_chunk; ++j) {
                    int node = 0;
                    for (;;) {
                        if (pos >= end) return CO3O_ERR_CORRUPT;
                        int nx = child[node][get_bit(words, pos++)];
                        if (nx == -1) return CO3O_ERR_CORRUPT;
                        if (nx < -1) { sym_put(sym, wide, elem + c0 + j, (uint32_t)(-nx - 2)); break; }
                        node = nx;
                    }
                }
                if (pos != end) return CO3O_ERR_CORRUPT;
            }
            if (((pos + 31) & ~(uint64_t)31) > chunk_offset[chunk + 1]) return CO3O_ERR_CORRUPT;
        }
        elem += seg_len[k];
    }
    return CO3O_OK;
}

/* ------------------------------------------------------------------------- */
/* PS side, eq. (aggregate hat) without the learning rate: the average of the */
/* users' reconstructed gradients (R8).  sym is [U][d] (row stride d), bias   */
/* is [U][nseg].                                                              */
int co3o_unpack(const uint32_t *words, uint64_t n_words, int nseg,
                const uint64_t *seg_len, const int32_t *seg_book,
                const uint8_t *len, const uint64_t *code, int A,
                const uint64_t *chunk_offset, const uint16_t *sub_bits,
                uint8_t *sym)
{
    return unpack_any(words, n_words, nseg, seg_len, seg_book, len, code, A, chunk_offset, sub_bits, sym, 0);
}
int co3o_unpack_w(const uint32_t *words, uint64_t n_words, int nseg,
                  const uint64_t *seg_len, const int32_t *seg_book,
                  const uint8_t *len, const uint64_t *code, int A,
                  const uint64_t *chunk_offset, const uint16_t *sub_bits,
                  uint16_t *sym)
{
    return unpack_any(words, n_words, nseg, seg_len, seg_book, len, code, A, chunk_offset, sub_bits, sym, 1);
}

/* ------------------------------------------------------------------------- */
static int aggregate_any(const void *sym, int wide, uint32_t U, uint64_t d, int nseg,
                         const uint64_t *seg_len, const int32_t *bias,
                         int exp_bits, int mant_bits, float *out)
{
    if (U == 0) return CO3O_ERR_ARG;
    double inv_u = 1.0 / (double)U;
    uint64_t elem = 0;
    for (int k = 0; k < nseg; ++k) {
        for (uint64_t i = elem; i < elem + seg_len[k]; ++i) {
            double acc = 0.0;
            for (uint32_t u = 0; u < U; ++u)
                acc += co3o_value(sym_get(sym, wide, (size_t)u * d + i), exp_bits, mant_bits,
                                  bias[(size_t)u * nseg + k]);
            out[i] = (float)(acc * inv_u);
        }
        elem += seg_len[k];
    }
    return (elem == d) ? CO3O_OK : CO3O_ERR_ARG;
}
int co3o_aggregate(const uint8_t *sym, uint32_t U, uint64_t d, int nseg,
                   const uint64_t *seg_len, const int32_t *bias,
                   int exp_bits, int mant_bits, float *out)
{
    return aggregate_any(sym, 0, U, d, nseg, seg_len, bias, exp_bits, mant_bits, out);
}
int co3o_aggregate_w(const uint16_t *sym, uint32_t U, uint64_t d, int nseg,
                     const uint64_t *seg_len, const int32_t *bias,
                     int exp_bits, int mant_bits, float *out)
{
    return aggregate_any(sym, 1, U, d, nseg, seg_len, bias, exp_bits, mant_bits, out);
}

/* The same average when the users' representatives carry a real-valued scale */
/* (reading R16): ghat = fl32(value(sym) c) with c = inv_gain[u][k], fp32.     */
static int aggregate_gain_any(const void *sym, int wide, uint32_t U, uint64_t d, int nseg,
                              const uint64_t *seg_len, const int32_t *bias, const float *inv_gain,
                              int exp_bits, int mant_bits, float *out)
{
    if (U == 0) return CO3O_ERR_ARG;
    double inv_u = 1.0 / (double)U;
    uint64_t elem = 0;
    for (int k = 0; k < nseg; ++k) {
        for (uint64_t i = elem; i < elem + seg_len[k]; ++i) {
            double acc = 0.0;
            for (uint32_t u = 0; u < U; ++u) {
                volatile float val = (float)co3o_value(sym_get(sym, wide, (size_t)u * d + i), exp_bits, mant_bits,
                                                       bias[(size_t)u * nseg + k]);
                volatile float q = val * inv_gain[(size_t)u * nseg + k];
                acc += (double)q;
            }
            out[i] = (float)(acc * inv_u);
        }
        elem += seg_len[k];
    }
    return (elem == d) ? CO3O_OK : CO3O_ERR_ARG;
}
int co3o_aggregate_gain(const uint8_t *sym, uint32_t U, uint64_t d, int nseg,
                        const uint64_t *seg_len, const int32_t *bias, const float *inv_gain,
                        int exp_bits, int mant_bits, float *out)
{
    return aggregate_gain_any(sym, 0, U, d, nseg, seg_len, bias, inv_gain, exp_bits, mant_bits, out);
}
int co3o_aggregate_gain_w(const uint16_t *sym, uint32_t U, uint64_t d, int nseg,
                          const uint64_t *seg_len, const int32_t *bias, const float *inv_gain,
                          int exp_bits, int mant_bits, float *out)
{
    return aggregate_gain_any(sym, 1, U, d, nseg, seg_len, bias, inv_gain, exp_bits, mant_bits, out);
}

/* ------------------------------------------------------------------------- */
/* PS model update, eq. (aggregate hat) / Algorithm 1 line 14:                */
/*   w_{t+1} = w_t - (eta / U) sum_u ghat^(u).                                */
/* The sum over u = 0..U-1 and the two products are taken in fp64 (sum, then  */
/* times 1/U, then times eta), the difference is rounded once to fp32.        */
/* ------------------------------------------------------------------------- */
static int model_update_any(const void *sym, int wide, uint32_t U, uint64_t d, int nseg,
                            const uint64_t *seg_len, const int32_t *bias,
                            int exp_bits, int mant_bits, float eta, const float *w, float *w_out)
{
    if (U == 0) return CO3O_ERR_ARG;
    double inv_u = 1.0 / (double)U;
    uint64_t elem = 0;
    for (int k = 0; k < nseg; ++k) {
        for (uint64_t i = elem; i < elem + seg_len[k]; ++i) {
            double acc = 0.0;
            for (uint32_t u = 0; u < U; ++u)
                acc += co3o_value(sym_get(sym, wide, (size_t)u * d + i), exp_bits, mant_bits,
                                  bias[(size_t)u * nseg + k]);
            w_out[i] = (float)((double)w[i] - (double)eta * (acc * inv_u));
        }
        elem += seg_len[k];
    }
    return (elem == d) ? CO3O_OK : CO3O_ERR_ARG;
}
int co3o_model_update(const uint8_t *sym, uint32_t U, uint64_t d, int nseg,
                      const uint64_t *seg_len, const int32_t *bias,
                      int exp_bits, int mant_bits, float eta, const float *w, float *w_out)
{
    return model_update_any(sym, 0, U, d, nseg, seg_len, bias, exp_bits, mant_bits, eta, w, w_out);
}
/* The same for alphabets of 9 to 12 bits (16-bit symbols). */
int co3o_model_update_w(const uint16_t *sym, uint32_t U, uint64_t d, int nseg,
                        const uint64_t *seg_len, const int32_t *bias,
                        int exp_bits, int mant_bits, float eta, const float *w, float *w_out)
{
    return model_update_any(sym, 1, U, d, nseg, seg_len, bias, exp_bits, mant_bits, eta, w, w_out);
}
