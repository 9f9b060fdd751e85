// Alphabets wider than one byte: formats with 9 to 12 symbol bits (1 + exp + mant), e.g. [1,5,6].
//
// The steps are those of the byte path (Algorithm 1 lines 8-10 and 13-14; Sec. IV-A (i)-(iii), Sec. II-B (iv))
// and the container is the same; symbols are 16-bit words and a code table has up to 4096 entries, too many
// for the per-wavefront LDS tables the byte kernels are built around.  These kernels keep the tables in
// device memory (they stay in the caches) and trade speed for simplicity: one element or one sub-chunk per
// lane, plain loops.  A fixed code without a symbol buffer ("single sweep" in the byte path) runs the same
// three steps here with the symbols kept in the workspace.
//
//   k_quantize_wide      v = g + gamma m, Q_fp, m' = v - ghat, symbol; symbol counts by global atomics
//   k_build_books_wide   Huffman code of a table on the device (same tie rule and canonical form as the host's)
//   k_chunk_bits_wide    code lengths summed per chunk
//   (k_scan_chunks of k_pack.hip gives the chunk offsets)
//   k_pack_wide          wavefront per chunk, lane per sub-chunk: lengths, wave prefix sum, codewords ORed into an
//                        LDS window at their bit offsets, window copied out
//   k_decode_wide        wavefront per (chunk, user), lane per sub-chunk: direct table for codes of up to 11 bits,
//                        canonical search by length above
//   k_aggregate_wide     the same decoder; values added to per-element fp64 sums in LDS, then averaged
#include "co3_internal.h"
#include "quantize_math.h"

namespace co3 {

constexpr int kWqThreads = 256;
constexpr int kWqPer = 4;                        // elements per thread
constexpr int kWqTile = kWqThreads * kWqPer;
constexpr int kWWaves = 4;                       // wavefronts per workgroup of the chunk kernels
constexpr int kWThreads = 64 * kWWaves;
constexpr int kWSymRow = kSub + 2;               // a sub-chunk's 64 staged symbols + pad (16-bit units)
constexpr int kWWin = 1024;                      // words of the pack window (8 bit/element per pass)
constexpr int kWbThreads = 1024;                 // threads of the table builder

__device__ inline uint32_t w_find_segment(const SegDev *segs, uint32_t nseg, uint64_t elem)
{
    uint32_t lo = 0, hi = nseg;  // segs[nseg].offset = d > elem
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (segs[mid].offset <= elem) lo = mid; else hi = mid;
    }
    return lo;
}

__device__ inline uint32_t w_find_chunk_segment(const SegDev *segs, uint32_t nseg, uint64_t chunk)
{
    uint32_t lo = 0, hi = nseg;  // segs[nseg].chunk_start = nchunks > chunk
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (segs[mid].chunk_start <= chunk) lo = mid; else hi = mid;
    }
    return lo;
}

__device__ inline void w_wave_sync_lds()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ inline uint32_t w_wave_sum(uint32_t x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

__device__ inline uint32_t w_wave_inclusive_scan(uint32_t x, uint32_t lane)
{
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t y = __shfl_up(x, o, 64);
        if ((int)lane >= o) x += y;
    }
    return x;
}

// Where chunk c lies: layer, first element, element count, code table within a user's set.
struct WChunk {
    uint32_t seg, n;
    uint64_t e0;
    uint32_t book;
};

__device__ inline WChunk w_chunk(const Layout &lay, uint64_t c, uint32_t u)
{
    WChunk k;
    k.seg = w_find_chunk_segment(lay.segs, lay.nseg, c);
    const SegDev sd = lay.segs[k.seg];
    k.e0 = sd.offset + (c - sd.chunk_start) * kChunk;
    const uint64_t left = sd.offset + sd.length - k.e0;
    k.n = left < (uint64_t)kChunk ? (uint32_t)left : (uint32_t)kChunk;
    k.book = (lay.per_user_books ? u * lay.books_per_user : 0u) + (uint32_t)sd.book;
    return k;
}

// ---- user side, step 1 ------------------------------------------------------------------------------------

__global__ __launch_bounds__(kWqThreads) void k_quantize_wide(Layout lay, const float *__restrict__ g, const float *m,
                                                              float *m_out, uint16_t *__restrict__ sym,
                                                              uint64_t sym_stride, uint64_t row_stride, float gamma,
                                                              uint64_t *__restrict__ hist_rep,
                                                              uint64_t *__restrict__ status)
{
    const uint32_t u = blockIdx.y;
    const uint64_t base = (uint64_t)blockIdx.x * kWqTile;
    const float *gu = g + (uint64_t)u * row_stride;
    const float *mu = m + (uint64_t)u * row_stride;
    float *mo = m_out + (uint64_t)u * row_stride;
    uint16_t *su = sym + (uint64_t)u * sym_stride;
    const uint32_t book_base = lay.per_user_books ? u * lay.books_per_user : 0u;
    uint64_t *hist = hist_rep + (uint64_t)(blockIdx.x % kHistGlobalRep) * lay.nbooks * lay.A;
    const uint32_t sign_shift = lay.E + lay.M;
    const uint32_t seg0 = w_find_segment(lay.segs, lay.nseg, base);
    uint32_t n_nonfinite = 0, n_clamped = 0;
    for (int k = 0; k < kWqPer; ++k) {
        const uint64_t i = base + (uint64_t)k * kWqThreads + threadIdx.x;
        if (i >= lay.d) break;
        uint32_t s_i = seg0;
        while (i >= lay.segs[s_i + 1].offset) ++s_i;   // ends: segs[nseg].offset = d > i
        const uint64_t pair = (uint64_t)u * lay.nseg + s_i;
        const int bias = lay.bias[pair];
        const QConst qc = make_qconst(lay.E, lay.M, bias);
        const float v = __fadd_rn(gu[i], __fmul_rn(gamma, mu[i]));
        const float y = __fmul_rn(v, lay.gain[2 * pair]);
        uint32_t s, flags;
        float q;
        quantize(y, qc, sign_shift, s, q, flags);
        q = __fmul_rn(q, lay.gain[2 * pair + 1]);
        mo[i] = (flags & 1u) ? 0.0f : __fsub_rn(v, q);
        n_nonfinite += flags & 1u;
        n_clamped += (flags >> 1) & 1u;
        su[i] = (uint16_t)s;
        atomicAdd(reinterpret_cast<unsigned long long *>(hist + (uint64_t)(book_base + lay.segs[s_i].book) * lay.A + s),
                  1ull);
    }
    if (n_nonfinite)
        atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_NONFINITE), (unsigned long long)n_nonfinite);
    if (n_clamped)
        atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CLAMPED), (unsigned long long)n_clamped);
}

__global__ __launch_bounds__(256) void k_reduce_hist_wide(const uint64_t *__restrict__ hist_rep,
                                                         uint64_t *__restrict__ hist, uint64_t n)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint64_t s = 0;
    for (int r = 0; r < kHistGlobalRep; ++r) s += hist_rep[(uint64_t)r * n + i];
    hist[i] = s;
}

__global__ void k_zero_wide(uint64_t *p, uint64_t n)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// ---- code tables ------------------------------------------------------------------------------------------

// One workgroup per table.  Dynamic LDS: node weights (2 A x 8 bytes) and parents (2 A x 4 bytes).
__global__ __launch_bounds__(kWbThreads) void k_build_books_wide(BookWide *__restrict__ books, uint32_t A,
                                                                const uint64_t *__restrict__ weights,
                                                                uint64_t *__restrict__ status)
{
    extern __shared__ uint64_t wb_smem[];
    uint64_t *nw = wb_smem;                                        // [2 A] sorted leaves, then internal nodes
    int *parent = reinterpret_cast<int *>(nw + 2 * (size_t)A);      // [2 A]
    __shared__ uint32_t cnt[65], off[65];
    __shared__ uint64_t first[65];
    __shared__ int err, s_n;
    __shared__ uint32_t s_maxlen;

    BookWide &B = books[blockIdx.x];
    const uint64_t *w = weights + (uint64_t)blockIdx.x * A;
    const uint32_t t = threadIdx.x;
    uint16_t *leaf_sym = B.sorted;   // sorted leaf -> symbol, until the canonical order replaces it

    if (t < 65) { cnt[t] = 0; off[t] = 0; first[t] = 0; }
    if (t == 0) { err = 0; s_maxlen = 0; s_n = 0; }
    for (uint32_t i = t; i < 2 * A; i += kWbThreads) parent[i] = -1;
    __syncthreads();
    int active = 0;
    for (uint32_t s = t; s < A; s += kWbThreads) {
        const uint64_t ws = w[s];
        if (ws == ~0ull) err = 1;    // 2^64 - 1 marks an exhausted queue in the merge: refused as a weight
        active += ws > 0 ? 1 : 0;
        B.len[s] = 0;
        B.code[s] = 0;
    }
    if (active) atomicAdd(&s_n, active);
    __syncthreads();
    const int nact = s_n;            // number of symbols with a weight

    // rank of every active symbol in (weight, symbol) order
    for (uint32_t s = t; s < A; s += kWbThreads) {
        const uint64_t ws = w[s];
        if (!ws) continue;
        int rank = 0;
        for (uint32_t j = 0; j < A; ++j) {
            const uint64_t wj = w[j];
            rank += (int)((wj != 0) & ((wj < ws) | ((wj == ws) & (j < s))));
        }
        nw[rank] = ws;
        leaf_sym[rank] = (uint16_t)s;
    }
    __syncthreads();

    if (t == 0 && nact >= 2 && !err) {
        const uint64_t kNone = ~0ull;
        int li = 0, ii = nact, made = nact;
        for (int step = 0; step < nact - 1; ++step) {
            int pick[2];
            uint64_t pw[2];
            for (int r = 0; r < 2; ++r) {
                const uint64_t lw = li < nact ? nw[li] : kNone, iw = ii < made ? nw[ii] : kNone;
                if (lw != kNone && (iw == kNone || lw <= iw)) { pick[r] = li++; pw[r] = lw; }
                else { pick[r] = ii++; pw[r] = iw; }
            }
            const uint64_t sum = pw[0] + pw[1];
            if (sum < pw[1] || sum == kNone) { err = 1; break; }  // the table's weights sum to 2^64 - 1 or more
            nw[made] = sum;
            parent[pick[0]] = made;
            parent[pick[1]] = made;
            ++made;
        }
    }
    __syncthreads();

    // depths of the leaves = code lengths
    for (int i = (int)t; i < nact; i += kWbThreads) {
        int depth = nact == 1 ? 1 : 0;
        for (int p = parent[i]; p >= 0 && depth <= CO3_MAX_CODE_LEN; p = parent[p]) ++depth;
        if (depth > CO3_MAX_CODE_LEN) err = 1;
        else B.len[leaf_sym[i]] = (uint8_t)depth;
    }
    __syncthreads();
    const bool bad = err != 0;
    if (bad) {
        for (uint32_t s = t; s < A; s += kWbThreads) B.len[s] = 0;
        if (t == 0) atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CODELEN), 1ull);
    }
    __syncthreads();
    for (uint32_t s = t; s < A; s += kWbThreads) {
        const uint32_t L = B.len[s];
        if (L) { atomicAdd(&cnt[L], 1u); atomicMax(&s_maxlen, L); }
    }
    __syncthreads();
    if (t == 0) {
        uint64_t code = 0;
        uint32_t o = 0;
        for (int l = 1; l <= 64; ++l) {
            code = (code + cnt[l - 1]) << 1;
            first[l] = code;
            off[l] = o;
            o += cnt[l];
        }
    }
    __syncthreads();
    // canonical order: rank among the symbols of the same length, ascending symbol
    for (uint32_t s = t; s < A; s += kWbThreads) {
        const uint32_t L = B.len[s];
        if (!L) continue;
        uint32_t rank = 0;
        for (uint32_t j = 0; j < s; ++j) rank += B.len[j] == L ? 1u : 0u;
        B.code[s] = first[L] + rank;
    }
    __syncthreads();  // every leaf_sym entry has been read (depths above); sorted[] may now take the canonical order
    for (uint32_t s = t; s < A; s += kWbThreads) {
        const uint32_t L = B.len[s];
        if (L) B.sorted[off[L] + (uint32_t)(B.code[s] - first[L])] = (uint16_t)s;
    }
    for (uint32_t i = (bad ? 0u : (uint32_t)nact) + t; i < A; i += kWbThreads) B.sorted[i] = 0;
    if (t < 65) { B.first[t] = first[t]; B.count[t] = cnt[t]; B.offset[t] = off[t]; }
    if (t == 0) { B.maxlen = s_maxlen; B.nactive = bad ? 0u : (uint32_t)nact; }
    __syncthreads();
    for (uint32_t idx = t; idx < (1u << kWideDecBits); idx += kWbThreads) {
        uint32_t e = 0;
        for (int l = 1; l <= kWideDecBits; ++l) {
            const uint32_t c = idx >> (kWideDecBits - l);
            const uint32_t f = (uint32_t)first[l];
            if (cnt[l] && c >= f && c - f < cnt[l]) {
                e = ((uint32_t)l << 16) | B.sorted[off[l] + (c - f)];
                break;
            }
        }
        B.dec[idx] = e;
    }
}

// ---- user side, steps 2 and 3 -------------------------------------------------------------------------------

__global__ __launch_bounds__(kWThreads) void k_chunk_bits_wide(Layout lay, const uint16_t *__restrict__ sym,
                                                              uint64_t sym_stride, const BookWide *__restrict__ books,
                                                              uint32_t *__restrict__ chunk_bits)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t c = (uint64_t)blockIdx.x * kWWaves + wave;
    const uint32_t u = blockIdx.y;
    if (c >= lay.nchunks) return;
    const WChunk k = w_chunk(lay, c, u);
    const uint8_t *len = books[k.book].len;
    const uint16_t *src = sym + (uint64_t)u * sym_stride + k.e0;
    uint32_t total = 0;
    for (uint32_t e = lane; e < k.n; e += 64) total += len[src[e] & (kWideMaxA - 1)];
    total = w_wave_sum(total);
    if (lane == 0) chunk_bits[(uint64_t)u * lay.nchunks + c] = total;
}

__global__ __launch_bounds__(kWThreads) void k_pack_wide(Layout lay, const uint16_t *__restrict__ sym, uint64_t sym_stride,
                                                        const BookWide *__restrict__ books,
                                                        const uint64_t *__restrict__ chunk_offset,
                                                        uint16_t *__restrict__ sub_bits, uint32_t *__restrict__ words,
                                                        uint64_t words_stride, uint64_t *__restrict__ status)
{
    __shared__ uint16_t s_sym_all[kWWaves][kSubsPerChunk * kWSymRow];
    __shared__ uint32_t s_win_all[kWWaves][kWWin + 1];
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t c = (uint64_t)blockIdx.x * kWWaves + wave;
    const uint32_t u = blockIdx.y;
    if (c >= lay.nchunks) return;  // whole wavefront; no workgroup barriers below
    uint16_t *s_sym = s_sym_all[wave];
    uint32_t *win = s_win_all[wave];
    const WChunk k = w_chunk(lay, c, u);
    const BookWide &book = books[k.book];
    const uint16_t *src = sym + (uint64_t)u * sym_stride + k.e0;
    for (uint32_t r = 0; r < (uint32_t)kSubsPerChunk; ++r) {   // element 64 r + lane -> row r
        const uint32_t e = lane + 64u * r;
        s_sym[r * kWSymRow + lane] = e < k.n ? (uint16_t)(src[e] & (kWideMaxA - 1)) : (uint16_t)0;
    }
    const uint64_t off = chunk_offset[(uint64_t)u * (lay.nchunks + 1) + c];
    w_wave_sync_lds();
    const int first = (int)lane * kSub;
    const int cnt = (int)k.n - first < 0 ? 0 : ((int)k.n - first > kSub ? kSub : (int)k.n - first);
    const uint16_t *row = s_sym + lane * kWSymRow;
    uint32_t bits = 0, nocode = 0;
    for (int j = 0; j < cnt; ++j) {
        const uint32_t L = book.len[row[j]];
        nocode += L == 0u ? 1u : 0u;
        bits += L;
    }
    if (nocode) atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_NOCODE), (unsigned long long)nocode);
    sub_bits[((uint64_t)u * lay.nchunks + c) * kSubsPerChunk + lane] = (uint16_t)bits;
    const uint32_t incl = w_wave_inclusive_scan(bits, lane);
    const uint32_t excl = incl - bits;
    const uint32_t chunk_total = __shfl(incl, 63, 64);
    const uint32_t nwords = (chunk_total + 31u) >> 5;
    const uint64_t off_words = off >> 5;
    if (off_words + nwords > words_stride) {
        if (lane == 0) atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CAPACITY), 1ull);
        return;
    }
    uint32_t *dst = words + (uint64_t)u * words_stride + off_words;
    for (uint32_t wbase = 0; wbase < nwords; wbase += kWWin) {
        const uint32_t wn = nwords - wbase < (uint32_t)kWWin ? nwords - wbase : (uint32_t)kWWin;
        for (uint32_t i = lane; i <= wn; i += 64) win[i] = 0u;
        w_wave_sync_lds();
        uint32_t wi = (excl >> 5) - wbase;  // window word receiving the next completed 32 bits (may start below the window)
        uint32_t np = excl & 31u;           // bits pending in acc (the leading np bits belong to earlier lanes)
        uint64_t acc = 0;
        auto append = [&](uint64_t code, uint32_t L) {  // L <= 32, np < 32
            acc = (acc << L) | code;
            np += L;
            if (np >= 32u) {
                np -= 32u;
                if (wi < wn) atomicOr(&win[wi], (uint32_t)(acc >> np));  // unsigned: false below the window
                ++wi;
            }
        };
        for (int j = 0; j < cnt; ++j) {
            const uint32_t s = row[j];
            uint32_t L = book.len[s];
            if (!L) continue;
            uint64_t code = book.code[s];
            if (L > 32u) {
                append(code >> 32, L - 32u);
                code &= 0xffffffffull;
                L = 32u;
            }
            append(code, L);
        }
        if (np && wi < wn) atomicOr(&win[wi], (uint32_t)(acc << (32u - np)));
        w_wave_sync_lds();
        for (uint32_t i = lane; i < wn; i += 64) dst[wbase + i] = win[i];
        w_wave_sync_lds();
    }
}

// ---- PS side ----------------------------------------------------------------------------------------------

// What the decoder keeps in LDS of one table.
struct WideTabs {
    uint32_t dec[1 << kWideDecBits];
    uint64_t first[65];
    uint32_t count[65];
    uint32_t offset[65];
    uint32_t maxlen;
    uint32_t pad;
};

__device__ inline void w_load_tabs(WideTabs *T, const BookWide &book, uint32_t t, uint32_t nthreads)
{
    for (uint32_t i = t; i < (1u << kWideDecBits); i += nthreads) T->dec[i] = book.dec[i];
    for (uint32_t i = t; i < 65u; i += nthreads) { T->first[i] = book.first[i]; T->count[i] = book.count[i]; T->offset[i] = book.offset[i]; }
    if (t == 0) { T->maxlen = book.maxlen > 64u ? 64u : book.maxlen; T->pad = 0; }
}

// The symbol whose codeword starts at bit `pos` of the chunk's nw words; len = 0 if none matches.  Reads nothing
// outside w[0 .. nw).
__device__ inline uint32_t w_decode_one(const uint32_t *__restrict__ w, uint32_t nw, uint32_t pos, const WideTabs *T,
                                        const uint16_t *__restrict__ sorted, uint32_t &len)
{
    const uint32_t i0 = pos >> 5, s0 = pos & 31u;
    const uint32_t w0 = i0 < nw ? w[i0] : 0u, w1 = i0 + 1u < nw ? w[i0 + 1u] : 0u, w2 = i0 + 2u < nw ? w[i0 + 2u] : 0u;
    uint64_t full = (((uint64_t)w0 << 32) | w1) << s0;
    if (s0) full |= (uint64_t)(w2 >> (32u - s0));
    const uint32_t e = T->dec[full >> (64 - kWideDecBits)];
    if (e) { len = e >> 16; return e & 0xffffu; }
    for (uint32_t L = kWideDecBits + 1; L <= T->maxlen; ++L) {
        const uint64_t cde = full >> (64u - L);
        if (T->count[L] && cde >= T->first[L] && cde - T->first[L] < (uint64_t)T->count[L]) {
            len = L;
            return sorted[(T->offset[L] + (uint32_t)(cde - T->first[L])) & (kWideMaxA - 1)];
        }
    }
    len = 0;
    return 0u;
}

// Index entries of chunk c of user u, checked as in the byte decoder.
struct WIndex {
    const uint32_t *w;
    uint32_t nw, sb;
    bool ok;
};

__device__ inline WIndex w_read_index(const Layout &lay, uint64_t c, uint32_t u, const uint32_t *__restrict__ words,
                                      uint64_t words_stride, const uint64_t *__restrict__ chunk_offset,
                                      const uint16_t *__restrict__ sub_bits, uint32_t lane)
{
    WIndex ix;
    const uint64_t off = chunk_offset[(uint64_t)u * (lay.nchunks + 1) + c];
    const uint64_t end = chunk_offset[(uint64_t)u * (lay.nchunks + 1) + c + 1];
    ix.sb = sub_bits[((uint64_t)u * lay.nchunks + c) * kSubsPerChunk + lane];
    ix.ok = !(off & 31u) && end >= off && (end >> 5) <= words_stride &&
            ((end - off) >> 5) <= (uint64_t)kChunk * CO3_MAX_CODE_LEN / 32;
    ix.nw = ix.ok ? (uint32_t)((end - off) >> 5) : 0u;
    ix.w = words + (uint64_t)u * words_stride + (ix.ok ? (off >> 5) : 0);
    return ix;
}

__global__ __launch_bounds__(kWThreads) void k_decode_wide(Layout lay, const uint32_t *__restrict__ words,
                                                          uint64_t words_stride,
                                                          const uint64_t *__restrict__ chunk_offset,
                                                          const uint16_t *__restrict__ sub_bits,
                                                          const BookWide *__restrict__ books, uint16_t *__restrict__ sym,
                                                          uint64_t sym_stride, float *__restrict__ q, uint64_t q_stride,
                                                          uint64_t *__restrict__ status)
{
    __shared__ WideTabs s_tabs[kWWaves];
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t c = blockIdx.x;
    const uint32_t u = blockIdx.y * kWWaves + wave;
    if (u >= lay.U) return;  // whole wavefront; wavefront-level synchronisation only below
    const WChunk k = w_chunk(lay, c, u);
    const BookWide &book = books[k.book];
    WideTabs *T = &s_tabs[wave];
    w_load_tabs(T, book, lane, 64);
    const WIndex ix = w_read_index(lay, c, u, words, words_stride, chunk_offset, sub_bits, lane);
    w_wave_sync_lds();
    const uint32_t p0 = w_wave_inclusive_scan(ix.sb, lane) - ix.sb;
    const int first = (int)lane * kSub;
    const int cnt = (int)k.n - first < 0 ? 0 : ((int)k.n - first > kSub ? kSub : (int)k.n - first);
    const uint64_t pair = (uint64_t)u * lay.nseg + k.seg;
    const int bias = lay.bias[pair];
    const float inv_gain = lay.gain[2 * pair + 1];
    uint32_t pos = p0;
    bool bad = false;
    for (int j = 0; j < cnt; ++j) {
        uint32_t len;
        const uint32_t s = w_decode_one(ix.w, ix.nw, pos, T, book.sorted, len);
        if (len == 0u) { bad = true; len = 1u; }
        pos += len;
        const uint64_t e = k.e0 + (uint64_t)first + (uint64_t)j;
        if (sym) sym[(uint64_t)u * sym_stride + e] = (uint16_t)s;
        if (q) q[(uint64_t)u * q_stride + e] = __fmul_rn(__uint_as_float(symbol_value_bits(s, lay.E, lay.M, bias)), inv_gain);
    }
    if (bad || pos - p0 != ix.sb || !ix.ok)
        atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CORRUPT), 1ull);
}

constexpr int kWAccStride = kSub + 1;
constexpr int kWAccWords = kSubsPerChunk * kWAccStride;

__global__ __launch_bounds__(kWThreads) void k_aggregate_wide(Layout lay, const uint32_t *__restrict__ words,
                                                             uint64_t words_stride,
                                                             const uint64_t *__restrict__ chunk_offset,
                                                             const uint16_t *__restrict__ sub_bits,
                                                             const BookWide *__restrict__ books, float *__restrict__ out,
                                                             float *__restrict__ model, float eta,
                                                             uint64_t *__restrict__ status)
{
    extern __shared__ uint64_t wa_smem[];
    double *s_acc = reinterpret_cast<double *>(wa_smem);                      // [64][kWAccStride]
    WideTabs *s_tabs = reinterpret_cast<WideTabs *>(s_acc + kWAccWords);      // [kWWaves]
    const uint32_t t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const uint64_t c = blockIdx.x;
    const WChunk k0 = w_chunk(lay, c, 0);
    for (uint32_t i = t; i < (uint32_t)kWAccWords; i += kWThreads) s_acc[i] = 0.0;
    __syncthreads();
    WideTabs *T = &s_tabs[wave];
    for (uint32_t u = wave; u < lay.U; u += kWWaves) {
        const WChunk k = w_chunk(lay, c, u);
        const BookWide &book = books[k.book];
        if (u == wave || lay.per_user_books) { w_wave_sync_lds(); w_load_tabs(T, book, lane, 64); }
        const WIndex ix = w_read_index(lay, c, u, words, words_stride, chunk_offset, sub_bits, lane);
        w_wave_sync_lds();
        const uint32_t p0 = w_wave_inclusive_scan(ix.sb, lane) - ix.sb;
        const int first = (int)lane * kSub;
        const int cnt = (int)k.n - first < 0 ? 0 : ((int)k.n - first > kSub ? kSub : (int)k.n - first);
        const uint64_t pair = (uint64_t)u * lay.nseg + k.seg;
        const int bias = lay.bias[pair];
        const float inv_gain = lay.gain[2 * pair + 1];
        double *acc = s_acc + lane * kWAccStride;
        uint32_t pos = p0;
        bool bad = false;
        for (int j = 0; j < cnt; ++j) {
            uint32_t len;
            const uint32_t s = w_decode_one(ix.w, ix.nw, pos, T, book.sorted, len);
            if (len == 0u) { bad = true; len = 1u; }
            pos += len;
            const float val = __fmul_rn(__uint_as_float(symbol_value_bits(s, lay.E, lay.M, bias)), inv_gain);
            __hip_atomic_fetch_add(&acc[j], (double)val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        if (bad || pos - p0 != ix.sb || !ix.ok)
            atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CORRUPT), 1ull);
    }
    __syncthreads();
    const double inv_u = 1.0 / (double)lay.U;
    const double eta64 = (double)eta;
    for (uint32_t e = t; e < k0.n; e += kWThreads) {
        const double avg = s_acc[(e >> 6) * kWAccStride + (e & 63u)] * inv_u;
        if (out) out[k0.e0 + e] = (float)avg;
        if (model) model[k0.e0 + e] = (float)((double)model[k0.e0 + e] - eta64 * avg);
    }
}

// ---- launchers ----------------------------------------------------------------------------------------------

static inline size_t w_up256(size_t x) { return (x + 255) & ~(size_t)255; }

// partial symbol counts, chunk sizes, and (for a fixed code without a symbol buffer) the symbols and their counts
size_t wide_workspace_bytes(const Layout &lay)
{
    const size_t sym_stride = (size_t)symbol_row_stride(lay.d);
    return w_up256((size_t)kHistGlobalRep * lay.nbooks * lay.A * sizeof(uint64_t)) +
           w_up256((size_t)lay.U * lay.nchunks * sizeof(uint32_t)) + w_up256((size_t)lay.nbooks * lay.A * sizeof(uint64_t)) +
           w_up256(sym_stride * lay.U * sizeof(uint16_t) + 32) + 512;
}

hipError_t launch_build_books_wide(BookWide *books, uint32_t nbooks, uint32_t A, const uint64_t *weights,
                                   uint64_t *status, hipStream_t s)
{
    if (nbooks == 0) return hipSuccess;
    const size_t lds = (size_t)2 * A * (sizeof(uint64_t) + sizeof(int));
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_build_books_wide),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    ProfScope prof(K_BUILD_BOOKS, s);
    hipLaunchKernelGGL(k_build_books_wide, dim3(nbooks), dim3(kWbThreads), lds, s, books, A, weights, status);
    return hipGetLastError();
}

hipError_t launch_encode_wide(const Layout &lay, const co3_encode_args &a, BookWide *books, void *workspace,
                              hipStream_t s)
{
    if (lay.U == 0) return hipSuccess;
    const uint64_t sym_stride = symbol_row_stride(lay.d);
    const uint64_t hist_n = (uint64_t)lay.nbooks * lay.A, hist_rep_n = (uint64_t)kHistGlobalRep * hist_n;
    uintptr_t p = (reinterpret_cast<uintptr_t>(workspace) + 255u) & ~(uintptr_t)255u;
    uint64_t *hist_rep = reinterpret_cast<uint64_t *>(p);
    p += w_up256(hist_rep_n * sizeof(uint64_t));
    uint32_t *chunk_bits = reinterpret_cast<uint32_t *>(p);
    p += w_up256((size_t)lay.U * lay.nchunks * sizeof(uint32_t));
    uint64_t *ws_hist = reinterpret_cast<uint64_t *>(p);
    p += w_up256(hist_n * sizeof(uint64_t));
    uint16_t *ws_sym = reinterpret_cast<uint16_t *>(p);
    // a fixed code without a symbol buffer: the symbols (and their counts, unused) stay in the workspace
    uint16_t *sym = a.symbols ? reinterpret_cast<uint16_t *>(a.symbols) : ws_sym;
    uint64_t *hist = a.hist ? a.hist : ws_hist;
    {
        ProfScope prof(K_ZERO, s);
        hipLaunchKernelGGL(k_zero_wide, dim3((uint32_t)((hist_rep_n + 255) / 256)), dim3(256), 0, s, hist_rep, hist_rep_n);
    }
    if (lay.d) {
        ProfScope prof(K_QUANTIZE, s);
        hipLaunchKernelGGL(k_quantize_wide, dim3((uint32_t)((lay.d + kWqTile - 1) / kWqTile), lay.U), dim3(kWqThreads), 0, s,
                           lay, a.g, a.m, a.m_out, sym, sym_stride, a.row_stride, a.gamma, hist_rep, a.status);
    }
    {
        ProfScope prof(K_REDUCE_HIST, s);
        hipLaunchKernelGGL(k_reduce_hist_wide, dim3((uint32_t)((hist_n + 255) / 256)), dim3(256), 0, s, hist_rep, hist, hist_n);
    }
    if (a.mode == CO3_BOOK_EMPIRICAL) {
        hipError_t e = launch_build_books_wide(books, lay.nbooks, lay.A, hist, a.status, s);
        if (e != hipSuccess) return e;
    }
    const uint32_t gx = (uint32_t)((lay.nchunks + kWWaves - 1) / kWWaves);
    if (lay.nchunks) {
        ProfScope prof(K_CHUNK_BITS, s);
        hipLaunchKernelGGL(k_chunk_bits_wide, dim3(gx, lay.U), dim3(kWThreads), 0, s, lay, sym, sym_stride, books, chunk_bits);
    }
    hipError_t e = launch_scan_chunks(lay, chunk_bits, a.chunk_offset, a.payload_bits, s);   // the byte path's scan
    if (e != hipSuccess) return e;
    if (lay.nchunks) {
        ProfScope prof(K_PACK, s);
        hipLaunchKernelGGL(k_pack_wide, dim3(gx, lay.U), dim3(kWThreads), 0, s, lay, sym, sym_stride, books,
                           a.chunk_offset, a.sub_bits, a.words, a.words_stride, a.status);
    }
    return hipGetLastError();
}

hipError_t launch_decode_wide(const Layout &lay, const co3_decode_args &a, const BookWide *books, hipStream_t s)
{
    if (lay.U == 0 || lay.nchunks == 0) return hipSuccess;
    const uint64_t sym_stride = symbol_row_stride(lay.d);
    ProfScope prof(K_DECODE, s);
    hipLaunchKernelGGL(k_decode_wide, dim3((uint32_t)lay.nchunks, (lay.U + kWWaves - 1) / kWWaves), dim3(kWThreads), 0, s,
                       lay, a.words, a.words_stride, a.chunk_offset, a.sub_bits, books,
                       reinterpret_cast<uint16_t *>(a.symbols), sym_stride, a.q, a.q_stride, a.status);
    return hipGetLastError();
}

hipError_t launch_aggregate_wide(const Layout &lay, const co3_aggregate_args &a, const BookWide *books, hipStream_t s)
{
    if (lay.U == 0 || lay.nchunks == 0) return hipSuccess;
    const size_t lds = (size_t)kWAccWords * sizeof(double) + (size_t)kWWaves * sizeof(WideTabs);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_aggregate_wide),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    ProfScope prof(K_AGGREGATE, s);
    hipLaunchKernelGGL(k_aggregate_wide, dim3((uint32_t)lay.nchunks), dim3(kWThreads), lds, s, lay, a.words,
                       a.words_stride, a.chunk_offset, a.sub_bits, books, a.out, a.model, a.eta, a.status);
    return hipGetLastError();
}

}  // namespace co3
