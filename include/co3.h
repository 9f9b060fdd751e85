/*
 * libco3 -- the per-iteration CO3 gradient codec on one AMD MI355X (gfx950).
 *
 * C ABI of the hot path of "Communication-Efficient Federated DNN Training: Convert,
 * Compress, Correct" (arXiv 2204.08211): error correction with memory decay, fp conversion,
 * element-wise Huffman coding, and the parameter server's decode + average.  U users are a
 * batch dimension on one GPU.  All the arithmetic runs in HIP kernels; there is no CPU
 * fallback.
 *
 * Conventions
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are plain
 *     host memory read (or written) before the call returns.
 *   - `stream` is a hipStream_t passed as void*; every kernel is enqueued on it and no call
 *     synchronises unless its comment says so.
 *   - every function returns a co3_status; data-dependent conditions (non-finite inputs,
 *     clamped inputs, symbols without a code, stream capacity, corrupt streams) are ADDED to
 *     the caller's device counter block `status` (CO3_STATUS_WORDS x uint64), which the caller
 *     clears and reads.
 *   - notation follows the paper: g gradient, m memory, gamma memory-decay coefficient,
 *     [sgn,exp,mant] float format, b = h_Hf(ghat) the binary string, r its length.
 */
#ifndef CO3_H
#define CO3_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CO3_CHUNK 4096u           /* elements per chunk (32-bit aligned unit of the stream) */
#define CO3_SUB 64u               /* elements per sub-chunk (unit one decoder lane owns)    */
#define CO3_SUBS_PER_CHUNK 64u
#define CO3_MAX_CODE_LEN 64
#define CO3_STATUS_WORDS 8

typedef enum {
    CO3_OK = 0,
    CO3_ERR_ARG = -1,       /* null pointer, bad size, misaligned buffer                    */
    CO3_ERR_FORMAT = -2,    /* [sgn,exp,mant] / bias outside what the library supports      */
    CO3_ERR_CAPACITY = -3,  /* workspace or stream buffer too small (host-detectable part)  */
    CO3_ERR_CODELEN = -4,   /* a Huffman code would need more than CO3_MAX_CODE_LEN bits     */
    CO3_ERR_CORRUPT = -5,
    CO3_ERR_HIP = -6        /* a HIP runtime call failed                                    */
} co3_status;

/* indices into the device counter block */
enum {
    CO3_STAT_NONFINITE = 0, /* inputs v = g + gamma m that are NaN or +-Inf                  */
    CO3_STAT_CLAMPED = 1,   /* finite inputs with |v| above the largest representative      */
    CO3_STAT_NOCODE = 2,    /* symbols met by the encoder that have no codeword             */
    CO3_STAT_CAPACITY = 3,  /* chunks not written because the stream buffer is too small    */
    CO3_STAT_CODELEN = 4,   /* code tables built on the device that needed > 64 bits        */
    CO3_STAT_CORRUPT = 5,   /* sub-chunks the decoder could not decode consistently         */
    CO3_STAT_STALLED = 6    /* workgroups of the single-sweep encoder whose bounded wait for
                             * the sizes of the preceding chunks ran out (their chunks are
                             * not written)                                                 */
};

/* Float format of Q_fp: one sign bit, exp_bits exponent bits, mant_bits mantissa bits
 * (Sec. IV-A (i); the sets M and E of Sec. V-B).  Requires exp_bits >= 2 and
 * 1 + exp_bits + mant_bits <= 12.  Up to 8 bits a symbol is one byte.  With 9 to 12 bits ("wide"
 * alphabets) a symbol is a 16-bit word: every `symbols` buffer below then holds uint16_t (its size is
 * co3_plan_symbols_bytes() all the same), the code tables have up to 4096 entries and the library
 * runs kernels of its own for them, in which a workgroup shares one copy of a table; a fixed code
 * without a symbol buffer is coded in the same three steps as with one, the symbols kept in the
 * workspace.                                                                                    */
typedef struct {
    int32_t exp_bits;
    int32_t mant_bits;
} co3_format;

/* One DNN layer of the flat gradient (Sec. II-D: layers are independent and differently
 * distributed; Sec. IV-A (ii): one code per layer).  Segments must be contiguous, in order,
 * and cover [0, d).  `codebook` selects the code table within a code-table set.            */
typedef struct {
    uint64_t offset;
    uint64_t length;
    int32_t codebook;
    int32_t reserved;
} co3_segment;

typedef struct co3_plan co3_plan;           /* layout of one round: library-owned           */
typedef struct co3_codebook co3_codebook;   /* a set of Huffman code tables: library-owned  */

/* ---- plan: problem statement of Sec. II-B (U users, d-dimensional gradients, the float
 * format and, per user and layer, the exponent bias) ------------------------------------
 * bias is host memory, [U][nseg]: the value exponent of exponent field f is f - bias, i.e.
 * the paper's c_scale = 2^b has b = (2^(exp_bits-1) - 1) - bias.  Required: bias <= 127 (the
 * smallest normal magnitude is a normal fp32) and (2^exp_bits - 2) - bias <= 100.
 * segments == NULL means one segment covering [0, d) with codebook 0.  per_user_books != 0
 * gives every user its own tables (table index u * books_per_user + segment.codebook)
 * instead of one table per layer shared by all users.
 * 1 <= U <= 65535.  Allocates small device tables; synchronises the device.  Not on the
 * per-iteration path: the paper holds the bias for several epochs (Sec. VI).               */
int co3_plan_create(co3_format format, uint32_t U, uint64_t d, uint32_t nseg,
                    const co3_segment *segments, const int32_t *bias, int32_t per_user_books,
                    co3_plan **out);
/* Replace the [U][nseg] bias table (host memory).  Synchronises `stream`.                  */
int co3_plan_set_bias(co3_plan *plan, const int32_t *bias, void *stream);
/* Real-valued scale (eq. (exp bias) of Sec. IV-A (i) lets b range over the reals, so c_scale = 2^b need not be
 * a power of two).  The integer bias carries the power-of-two part; this call adds, per user and layer, a
 * gain s applied to the input of the conversion and its reciprocal c applied to the representative, in fp32:
 *   y = fl32(v s),  symbol = code of Q_fp(y),  ghat = fl32(value(symbol) c),  m' = fl32(v - ghat),
 * so that the representative set becomes {c x : x in X}; m' is then no longer the exact difference.  The PS side
 * (co3_decode's q, co3_ps_aggregate) forms ghat the same way.  gain, inv_gain: host [U][nseg], positive normal
 * fp32 numbers, the caller supplying the pair (typically inv_gain = 2^(b - round(b)), gain = 1 / inv_gain); both
 * NULL restores 1.  Non-finite and clamped inputs are judged on y.  Not combined with CO3_ROUND_STOCHASTIC
 * (co3_encode then returns CO3_ERR_ARG).  Synchronises `stream`.                                              */
int co3_plan_set_gain(co3_plan *plan, const float *gain, const float *inv_gain, void *stream);
void co3_plan_destroy(co3_plan *plan);
uint64_t co3_plan_num_chunks(const co3_plan *plan);     /* chunks per user                  */
uint32_t co3_plan_num_books(const co3_plan *plan);      /* tables in a matching set         */
uint32_t co3_plan_alphabet(const co3_plan *plan);       /* A = 2^(1+exp_bits+mant_bits)     */
/* bytes of the `symbols` buffer of co3_encode_args / co3_decode_args: U rows of d symbols, each row
 * padded to a multiple of 128 symbols, plus 16 symbols; one byte per symbol (two for wide alphabets) */
size_t co3_plan_symbols_bytes(const co3_plan *plan);
/* bytes of the `workspace` buffer of co3_encode_args                                       */
size_t co3_plan_workspace_bytes(const co3_plan *plan);
/* words per user that hold any stream whose longest codeword has max_code_len bits         */
uint64_t co3_plan_stream_words(const co3_plan *plan, uint32_t max_code_len);

/* ---- code tables: h_Hf of Sec. IV-A (ii) ------------------------------------------------
 * co3_build_codebook: Huffman codes for nbooks tables from integer weights (host memory,
 * [nbooks][A], weight 0 = symbol has no code); weights == NULL only allocates the set, to be
 * filled by co3_build_codebook_device.  Ties are broken by (weight, key) with leaf key =
 * symbol and internal key = A + creation order; codes are canonical by (length, symbol).
 * Runs on the host, uploads the tables, synchronises the device.
 * Errors: CO3_ERR_CODELEN if a code would exceed 64 bits, CO3_ERR_ARG if a table's weights
 * sum to 2^64 - 1 or more.                                                                  */
int co3_build_codebook(co3_format format, uint32_t nbooks, const uint64_t *weights,
                       co3_codebook **out);
/* Rebuild every table of `books` on the device from device weights [nbooks][A] (e.g. the
 * histogram co3_encode wrote), with no host round trip.  Tables needing more than 64 bits
 * are left empty and counted in status[CO3_STAT_CODELEN].                                  */
int co3_build_codebook_device(co3_codebook *books, const uint64_t *weights, uint64_t *status,
                              void *stream);
/* Copy one table to host memory (len[A], code[A]) for inspection.  Synchronises `stream`.  */
int co3_codebook_export(const co3_codebook *books, uint32_t book, uint8_t *len, uint64_t *code,
                        void *stream);
uint32_t co3_codebook_num_books(const co3_codebook *books);
void co3_codebook_destroy(co3_codebook *books);

/* Integer weights for co3_build_codebook when the corrected gradient g + gamma m of a layer is
 * modelled as GenNorm(mu, alpha, beta) (Sec. III eq. (gennorm); Sec. IV-A (ii): the Huffman code
 * is designed from that model).  weights is host memory, A entries: every symbol Q_fp can
 * produce gets max(1, floor(p * 2^40)), p the model probability that Q_fp yields it; the other
 * bit patterns (top exponent field, negative zero) get 0.  Host arithmetic, no GPU involved.
 * Errors: CO3_ERR_ARG for alpha <= 0, beta <= 0 or a non-finite mu; CO3_ERR_FORMAT.          */
int co3_gennorm_weights(co3_format format, int32_t bias, double mu, double alpha, double beta,
                        uint64_t *weights);

/* ---- the GenNorm model from the data (Sec. III eq. (kurtosis); Sec. IV-A (ii); Sec. VI) -----
 * co3_gennorm_fit: for every user and layer, the GenNorm(mu, alpha, beta) whose mean, variance
 * and kurtosis (eq. (kurtosis)) equal those of the sample v = g + gamma m: one read sweep over g
 * and m (fp64 sums of v, v^2, v^3, v^4 in a fixed order), then beta from the kurtosis by bisection
 * on [0.1, 64] (clamped) and alpha from the variance.  params is device memory [U][nseg]; an empty
 * or constant layer (variance below 2^-40 of the mean square) gets alpha = beta = 0.
 * workspace: device, co3_plan_fit_workspace_bytes().
 * The paper fits once and holds the parameters for several epochs; so does a caller of this.
 * co3_model_weights_device: integer Huffman weights (device, [num_books][A]) of the model code
 * for those parameters: a table's source is the mixture of the quantized models of the (user,
 * layer) pairs it serves, weighted by their element counts; every symbol Q_fp can produce gets
 * max(1, floor(p * 2^40)), the others 0.  Feed them to co3_build_codebook_device.             */
typedef struct {
    double mu, alpha, beta;
    double kurtosis;         /* the sample's m4 / m2^2                                        */
} co3_gennorm_params;
size_t co3_plan_fit_workspace_bytes(const co3_plan *plan);
int co3_gennorm_fit(const co3_plan *plan, const float *g, const float *m, uint64_t row_stride,
                    float gamma, co3_gennorm_params *params, void *workspace,
                    size_t workspace_bytes, void *stream);
int co3_model_weights_device(const co3_plan *plan, const co3_gennorm_params *params,
                             uint64_t *weights, void *stream);
/* Exponent bias from the model: eq. (exp bias) of Sec. IV-A (i), b_t = argmin_b E|Q_fp(G) - G|^2,
 * with b restricted to the integers (power-of-two scale) and G ~ GenNorm(params): the expectation
 * in closed form (partial moments of GenNorm through incomplete gamma functions) for every bias
 * the library supports; errors within 1e-9 (relative) of the minimum count as equal and the
 * smallest such bias is taken; a layer without a model (alpha = 0) gets 2^(exp_bits-1) - 1.
 * bias: device [U][nseg] (out); error: device [U][nseg] expected squared errors, or NULL;
 * workspace: device, co3_plan_bias_workspace_bytes().
 * co3_plan_set_bias_device installs a device bias table in the plan (device-to-device copy on
 * `stream`, no synchronisation); its values must be in the supported range, as the ones written
 * by co3_model_bias_device are.  co3_bias_from_model is the same argmin for one parameter triple
 * on the host.                                                                               */
size_t co3_plan_bias_workspace_bytes(const co3_plan *plan);
int co3_model_bias_device(const co3_plan *plan, const co3_gennorm_params *params, int32_t *bias,
                          double *error, void *workspace, size_t workspace_bytes, void *stream);
int co3_plan_set_bias_device(co3_plan *plan, const int32_t *bias, void *stream);
int co3_bias_from_model(co3_format format, double mu, double alpha, double beta, int32_t *bias,
                        double *error);
/* eq. (exp bias) of Sec. IV-A (i) with b ranging over the reals, for one parameter triple, on the host: the
 * integer bias that carries the power-of-two part of c_scale = 2^b and the fp32 pair (gain, inv_gain) for
 * co3_plan_set_gain that carries the rest, inv_gain = fl32(2^t) with t in [-1/2, 1/2], gain = fl32(1 / inv_gain).
 * The same closed-form expectation as co3_bias_from_model, scanned in steps of 1/16 binade over one and a half
 * binades to either side of the integer optimum and refined by a golden-section search.  Where no real scale
 * lowers the expected error by more than 1e-9 (relative) - formats with many binades, layers without a model -
 * the integer result is returned with gain = inv_gain = 1.  error (may be NULL): the expected squared error of
 * the returned triple.                                                                                       */
int co3_scale_from_model(co3_format format, double mu, double alpha, double beta, int32_t *bias, float *gain,
                         float *inv_gain, double *error);

/* The same search on the device for every (user, layer) of a plan, from fitted parameters: first the integer
 * argmin as in co3_model_bias_device, then scan and golden-section search over the real scale as in
 * co3_scale_from_model, every expected error summed over the symbols' cells by one workgroup in a fixed order.
 * bias: device [U][nseg] (out); gain_pairs: device [U][nseg][2] (out), (gain, inv_gain) per pair, (1, 1) where
 * the integer result stays; error: device [U][nseg] expected squared errors of the returned triples, or NULL;
 * workspace: device, co3_plan_scale_workspace_bytes().  No synchronisation; no host copy of the results.
 * co3_plan_set_gain_device installs such a table of pairs in the plan (device-to-device copy on `stream`; the
 * values must be positive normal numbers, as the ones written here are); the plan then counts as carrying a
 * scale - the stochastic conversion is refused - until co3_plan_set_gain(plan, NULL, NULL, ...) removes it.   */
size_t co3_plan_scale_workspace_bytes(const co3_plan *plan);
int co3_model_scale_device(const co3_plan *plan, const co3_gennorm_params *params, int32_t *bias, float *gain_pairs,
                           double *error, void *workspace, size_t workspace_bytes, void *stream);
int co3_plan_set_gain_device(co3_plan *plan, const float *gain_pairs, void *stream);

/* ---- user side: Algorithm 1 lines 8-10 for all U users -----------------------------------
 * v = g + gamma m (eq. (f_error_fb)), ghat = Q_fp(v), m' = v - ghat, b = h_Hf(ghat).
 * mode CO3_BOOK_FIXED encodes with `books` as they are (a code designed beforehand, e.g. from
 * the GenNorm model); CO3_BOOK_EMPIRICAL first rebuilds `books` on the device from this
 * round's symbol histogram.
 * In mode CO3_BOOK_FIXED `symbols` may be NULL: the library then runs the single-sweep encoder,
 * in which the symbols never reach device memory (12 bytes of traffic per element plus the
 * stream).  `hist` may be NULL too; if it is given, the sweep also counts this round's symbols
 * per code table (e.g. to design the next round's code from them while this round's is held),
 * at a lower occupancy of the kernel.                                                         */
enum { CO3_BOOK_FIXED = 0, CO3_BOOK_EMPIRICAL = 1 };
/* Q_fp picks the closest representative (Sec. IV-A (i)), or, as the stochastic mapping Sec. II-B
 * (ii) allows (non-subtractive dither), the upper of the two neighbours with probability
 * (|v| - lo) / (hi - lo): a uniform integer dither is added to the position of |v| between them
 * (its low 23 - mant_bits fp32 pattern bits in the normal range; 24 fractional bits of
 * |v| / 2^(1 - bias - mant_bits) in the zero/subnormal row) and the result truncated.  Element i
 * of user u uses word i mod 4 of Philox4x32-10(counter = (i/4 low, i/4 high, u, 0), key = seed). */
enum { CO3_ROUND_NEAREST = 0, CO3_ROUND_STOCHASTIC = 1 };

typedef struct {
    const float *g;          /* device [U][row_stride] gradients; 16-byte aligned            */
    const float *m;          /* device [U][row_stride] memory m_{t-1}                        */
    float *m_out;            /* device [U][row_stride] memory m_t; may equal m               */
    uint64_t row_stride;     /* elements between users, >= d, multiple of 4 (a multiple of  */
                             /* 32 keeps the 16 KB chunks on 128-byte lines: a few % faster) */
    float gamma;             /* memory-decay coefficient                                     */
    int32_t mode;            /* CO3_BOOK_FIXED or CO3_BOOK_EMPIRICAL                         */
    co3_codebook *books;     /* set with co3_plan_num_books() tables                         */
    uint8_t *symbols;        /* device, co3_plan_symbols_bytes(): [U][d] symbols (out);      */
                             /* uint16_t words for wide alphabets                            */
    uint64_t *hist;          /* device [num_books][A] symbol counts (out; cleared here)      */
                             /* (symbols NULL, fixed code: the single-sweep encoder; hist    */
                             /* is then optional)                                            */
    uint32_t *words;         /* device [U][words_stride] streams (out)                       */
    uint64_t words_stride;   /* capacity of one user's stream in 32-bit words                */
    uint64_t *chunk_offset;  /* device [U][num_chunks+1] bit offsets of the chunks (out)     */
    uint16_t *sub_bits;      /* device [U][num_chunks*64] bits per sub-chunk (out); may be   */
                             /* NULL when d = 0                                              */
    uint64_t *payload_bits;  /* device [U]: r = sum of codeword lengths (out)                */
    uint64_t *status;        /* device [CO3_STATUS_WORDS] counters (added to)                */
    void *workspace;         /* device, co3_plan_workspace_bytes()                           */
    size_t workspace_bytes;
    int32_t rounding;        /* CO3_ROUND_NEAREST or CO3_ROUND_STOCHASTIC                    */
    int32_t reserved;
    uint64_t seed;           /* key of the dither generator (vary it from round to round)    */
} co3_encode_args;

/* Enqueues the whole user side on `stream`.  Stream words beyond a user's last chunk are not
 * written.  A chunk that does not fit words_stride is skipped and counted.                  */
int co3_encode(const co3_plan *plan, const co3_encode_args *args, void *stream);

/* co3_encode for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and same results as co3_encode, but `workspace` / `workspace_bytes` are ignored: the
 * partial histograms, per-chunk sizes, ticket counters and look-back entries live in a static
 * device array of CO3_STATIC_SCRATCH_BYTES that is part of the library (every GPU the library runs
 * on holds one copy until the process ends; its address on a device is resolved when a plan is
 * created there).  The call allocates nothing.  The static array has room for the encoders' smallest
 * workspace only (about 4 bytes per user and chunk plus the partial histograms, not the per-chunk
 * symbol counts co3_plan_workspace_bytes() also provides for, which spare the three-step encoder a
 * sweep): a plan whose smallest workspace exceeds CO3_STATIC_SCRATCH_BYTES is refused with
 * CO3_ERR_CAPACITY before anything is launched; between
 * co3_profile_begin() and co3_profile_end() (event timing creates events) it returns CO3_ERR_ARG.
 * All calls on one GPU share that array: what must start at zero is cleared by the call itself,
 * but two calls that overlap on one GPU (different streams, or threads) race -- serialise them.   */
#define CO3_STATIC_SCRATCH_BYTES (8u << 20)
int co3_encode_static(const co3_plan *plan, const co3_encode_args *args, void *stream);

/* ---- PS side: Algorithm 1 lines 13-14 ----------------------------------------------------*/
typedef struct {
    const uint32_t *words;        /* device [U][words_stride]                                */
    uint64_t words_stride;
    const uint64_t *chunk_offset; /* device [U][num_chunks+1]                                */
    const uint16_t *sub_bits;     /* device [U][num_chunks*64]                               */
    const co3_codebook *books;
    uint8_t *symbols;             /* device, co3_plan_symbols_bytes(), or NULL (out);        */
                                  /* uint16_t words for wide alphabets                       */
    float *q;                     /* device [U][q_stride] reconstructed ghat, or NULL (out)  */
    uint64_t q_stride;
    uint64_t *status;
} co3_decode_args;

/* h_Hf^-1 (Sec. II-B (iii): the mapping h is invertible): symbols and/or values of every
 * user's stream.  Never reads outside [0, words_stride) of a user's stream; inconsistent
 * sub-chunks are counted in status[CO3_STAT_CORRUPT] and their outputs are unspecified.     */
int co3_decode(const co3_plan *plan, const co3_decode_args *args, void *stream);

typedef struct {
    const uint32_t *words;
    uint64_t words_stride;
    const uint64_t *chunk_offset;
    const uint16_t *sub_bits;
    const co3_codebook *books;
    float *out;                   /* device [d]: (1/U) sum_u ghat^(u); may be NULL if model is set */
    uint64_t *status;
    float *model;                 /* device [d] or NULL: w, updated in place (see below)          */
    float eta;                    /* learning rate of the update                                  */
    int32_t reserved;
} co3_aggregate_args;

/* Decode all U streams and average them (eq. (aggregate hat) without the learning rate):
 * out[i] = fl32((sum over u = 0..U-1, in fp64, of ghat_i^(u)) * (1.0 / U)).
 * With `model`, also the PS model update of eq. (aggregate hat) / Algorithm 1 line 14 in the same
 * pass: model[i] = fl32(model[i] - eta * ((sum over u) * (1.0 / U))), products and difference in
 * fp64, one rounding.  With five or more users the fp64 sums are formed by atomic additions in
 * whatever order the wavefronts arrive.  The addends are representatives, so the sum is exact,
 * and independent of that order, whenever (2^exp_bits - 2) + mant_bits + 1 + (largest minus
 * smallest bias of the layer over the users) + log2 U <= 53 (add 23 - mant_bits for a plan that
 * carries a gain); beyond that the last bit of a sum may depend on the order.                 */
int co3_ps_aggregate(const co3_plan *plan, const co3_aggregate_args *args, void *stream);

/* ---- measurement aid ---------------------------------------------------------------------
 * Between co3_profile_begin() and co3_profile_end() every kernel the library launches is
 * bracketed by two HIP events recorded on the stream it is launched on.  co3_profile_end
 * synchronises the device and returns, per kernel name, the summed elapsed time and the
 * number of launches (at most `capacity` entries; *count gets the number written).         */
typedef struct {
    char name[32];
    double total_ms;
    uint64_t launches;
} co3_kernel_time;
int co3_profile_begin(void);
int co3_profile_end(co3_kernel_time *out, uint32_t capacity, uint32_t *count);

/* The single-sweep encoder waits for the sizes of the chunks ahead of a workgroup by polling; the
 * wait is bounded by `polls` re-reads per predecessor entry (default CO3_LOOKBACK_POLLS_DEFAULT,
 * far more than any wait that ends).  A workgroup whose bound runs out writes no stream words,
 * leaves its chunk_offset entries untouched and is counted in status[CO3_STAT_STALLED]; so are all
 * later workgroups of that user.  m_out, sub_bits and payload_bits are complete all the same.
 * polls = 0 gives up at the first entry that is not there yet (a way to exercise that path from
 * the host).  Process-wide; applies to calls of co3_encode made afterwards.                    */
#define CO3_LOOKBACK_POLLS_DEFAULT (1u << 20)
void co3_set_lookback_polls(uint32_t polls);

/* Human-readable name of a status code.                                                     */
const char *co3_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* CO3_H */
