// Alphabets wider than one byte: formats with 9 to 12 symbol bits (1 + exp + mant), e.g. [1,5,6].
//
// The steps are those of the byte path (Algorithm 1 lines 8-10 and 13-14; Sec. IV-A (i)-(iii), Sec. II-B (iv))
// and the container is the same; symbols are 16-bit words and a code table has up to 4096 entries, too many
// for the per-wavefront LDS tables the byte kernels are built around: here a workgroup shares one copy of the
// table of the layer it works on, and falls back to the table in device memory where its range of the vector
// crosses into a layer with another table.  A fixed code without a symbol buffer ("single sweep" in the byte
// path) runs the same three steps here with the symbols kept in the workspace.
//
//   k_quantize_wide      v = g + gamma m, Q_fp, m' = v - ghat, symbol; symbol counts in an LDS table per workgroup
//                        (and, for a held code on layers that start on its tile grid, the chunks' coded sizes)
//   k_build_books_wide   Huffman code of a table on the device (same tie rule and canonical form as the host's):
//                        bitonic sort, two-queue merge, depths, canonical ranks from ballots
//   k_chunk_bits_wide    code lengths summed per chunk, lengths in LDS
//   (k_scan_chunks of k_pack.hip gives the chunk offsets)
//   k_pack_wide          wavefront per chunk, lane per sub-chunk with its 64 symbols in registers: lengths, wave
//                        prefix sum, codewords ORed into an LDS window at their bit offsets, window copied out
//   k_decode_wide        wavefront per (chunk, user), lane per sub-chunk: prefix table for codes of up to 12 bits,
//                        second-level tables over the next 5 bits under the first 128 prefixes of longer codes,
//                        the rest by their value among the per-length bounds of the canonical code
//   k_aggregate_wide     the same decoder; values added to per-element fp64 sums in LDS, then averaged
#include "co3_internal.h"
#include "quantize_math.h"

namespace co3 {

constexpr int kWqThreads = 256;
constexpr int kWqPer = 8;                        // elements per thread and tile
constexpr int kWqTile = kWqThreads * kWqPer;
constexpr int kWWaves = 4;                       // wavefronts per workgroup of the chunk kernels
constexpr int kWThreads = 64 * kWWaves;
constexpr int kWSymRow = kSub + 2;               // a sub-chunk's 64 staged symbols + pad (16-bit units)
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

// A workgroup takes kWqTiles consecutive tiles of one user and counts their symbols in an LDS table of the code
// table in use (A entries), which it adds to one of the global partial tables when the code table changes (a layer
// with another table begins) and at its end; the few elements of a tile that belong to another table than the
// tile's first element are counted in global memory directly.
constexpr int kWqTiles = 32;
typedef float wf4 __attribute__((ext_vector_type(4)));
typedef uint32_t wu2 __attribute__((ext_vector_type(2)));
// kSR: the stochastic conversion (dither from Philox words of (element, user, seed)) instead of the closest
// representative.
// kBits: the code is known beforehand and every layer starts at a multiple of the tile (lay.tile_aligned), so
// that a tile lies in one chunk: the chunks' coded sizes are summed here (chunk_bits, zero on entry) and the
// sweep over the symbols that would count them is not needed.
template <bool kSR, bool kBits>
__global__ __launch_bounds__(kWqThreads) void k_quantize_wide(Layout lay, const float *__restrict__ g, const float *m,
                                                              float *m_out, uint16_t *__restrict__ sym,
                                                              uint64_t sym_stride, uint64_t row_stride, float gamma,
                                                              uint64_t seed, uint64_t *__restrict__ hist_rep,
                                                              const BookWide *__restrict__ books,
                                                              uint32_t *__restrict__ chunk_bits,
                                                              uint64_t *__restrict__ status)
{
    __shared__ uint32_t s_hist[kWideMaxA];
    __shared__ uint32_t s_len4[kBits ? kWideMaxA / 4 : 1];   // the code lengths of the table in use, four per word
    const uint8_t *s_len8 = reinterpret_cast<const uint8_t *>(s_len4);
    const uint32_t u = blockIdx.y;
    const float *gu = g + (uint64_t)u * row_stride;
    const float *mu = m + (uint64_t)u * row_stride;
    float *mo = m_out + (uint64_t)u * row_stride;
    uint16_t *su = sym + (uint64_t)u * sym_stride;
    const uint32_t book_base = lay.per_user_books ? u * lay.books_per_user : 0u;
    uint64_t *hist = hist_rep + (uint64_t)(blockIdx.x % kHistGlobalRep) * lay.nbooks * lay.A;
    const uint32_t sign_shift = lay.E + lay.M;
    uint32_t n_nonfinite = 0, n_clamped = 0;
    for (uint32_t i = threadIdx.x; i < lay.A; i += kWqThreads) s_hist[i] = 0u;
    __syncthreads();
    auto flush = [&](uint32_t book) {   // between two workgroup barriers
        for (uint32_t i = threadIdx.x; i < lay.A; i += kWqThreads) {
            const uint32_t c = s_hist[i];
            if (c) atomicAdd(reinterpret_cast<unsigned long long *>(hist + (uint64_t)book * lay.A + i), (unsigned long long)c);
            s_hist[i] = 0u;
        }
    };
    uint32_t cur_book = 0xffffffffu;   // workgroup-uniform, like the layer of the tile's first element:
    uint32_t seg0 = 0, tile_book = 0;
    uint64_t seg_end = 0;              // where that layer ends (0: none looked up yet)
    uint64_t seg_off = 0, seg_chunk0 = 0;   // where it starts, and its first chunk
    int bias0 = 0;
    QConst qc0 = make_qconst(lay.E, lay.M, 0);
    float gain0 = 1.0f, inv_gain0 = 1.0f;
    for (int tile = 0; tile < kWqTiles; ++tile) {
        const uint64_t base = ((uint64_t)blockIdx.x * kWqTiles + (uint64_t)tile) * kWqTile;
        if (base >= lay.d) break;      // workgroup-uniform
        if (base >= seg_end) {         // the tile starts in another layer than the last one did: look it up
            seg0 = w_find_segment(lay.segs, lay.nseg, base);
            seg_end = lay.segs[seg0 + 1].offset;
            seg_off = lay.segs[seg0].offset;
            seg_chunk0 = lay.segs[seg0].chunk_start;
            tile_book = book_base + (uint32_t)lay.segs[seg0].book;
            const uint64_t pair0 = (uint64_t)u * lay.nseg + seg0;
            bias0 = lay.bias[pair0];
            qc0 = make_qconst(lay.E, lay.M, bias0);
            gain0 = lay.gain[2 * pair0];
            inv_gain0 = lay.gain[2 * pair0 + 1];
        }
        if (tile_book != cur_book) {
            __syncthreads();
            if (cur_book != 0xffffffffu) flush(cur_book);
            if constexpr (kBits) {
                const uint32_t *len4 = reinterpret_cast<const uint32_t *>(books[tile_book].len);
                for (uint32_t i = threadIdx.x; i < (uint32_t)kWideMaxA / 4; i += kWqThreads) s_len4[i] = len4[i];
            }
            __syncthreads();
            cur_book = tile_book;
        }
        uint32_t tile_bits = 0;        // code lengths of this thread's elements of the tile
        auto add_tile_bits = [&]() {   // by every wavefront, once per tile
            if constexpr (kBits) {
                const uint32_t sum = w_wave_sum(tile_bits);
                if ((threadIdx.x & 63u) == 0u && sum)
                    atomicAdd(&chunk_bits[(uint64_t)u * lay.nchunks + seg_chunk0 + ((base - seg_off) >> 12)], sum);
            }
        };
        // the scale and the quantizer's constants of the tile's first layer serve the whole tile unless it
        // crosses into the next layer
        const uint64_t tile_end = base + kWqTile < lay.d ? base + kWqTile : lay.d;
        const bool one_layer = tile_end <= seg_end;
        if (one_layer && base + kWqTile <= lay.d) {
            // a whole tile of one layer (rows and tiles start on 16-byte boundaries): thread t takes elements
            // 4 t .. 4 t + 3 of each half, 16-byte loads and stores, four symbols per 8-byte store
            wf4 gq[kWqPer / 4], mq[kWqPer / 4];
#pragma unroll
            for (int k = 0; k < kWqPer / 4; ++k) {
                const uint64_t i = base + (uint64_t)k * (kWqThreads * 4) + threadIdx.x * 4;
                gq[k] = __builtin_nontemporal_load(reinterpret_cast<const wf4 *>(gu + i));
                mq[k] = __builtin_nontemporal_load(reinterpret_cast<const wf4 *>(mu + i));
            }
#pragma unroll
            for (int k = 0; k < kWqPer / 4; ++k) {
                const uint64_t i = base + (uint64_t)k * (kWqThreads * 4) + threadIdx.x * 4;
                wf4 eo;
                uint32_t sp[4];
                Philox4 rw;
                if constexpr (kSR) rw = element_random_words(i, u, seed);   // i is a multiple of 4
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float v = __fadd_rn(gq[k][j], __fmul_rn(gamma, mq[k][j]));
                    const float y = __fmul_rn(v, gain0);
                    uint32_t s, flags;
                    float q;
                    if constexpr (kSR) quantize_stochastic(y, qc0, lay.E, lay.M, bias0, sign_shift, rw.w[j], s, q, flags);
                    else quantize(y, qc0, sign_shift, s, q, flags);
                    q = __fmul_rn(q, inv_gain0);
                    eo[j] = (flags & 1u) ? 0.0f : __fsub_rn(v, q);
                    n_nonfinite += flags & 1u;
                    n_clamped += (flags >> 1) & 1u;
                    sp[j] = s;
                    atomicAdd(&s_hist[s & (kWideMaxA - 1)], 1u);
                    if constexpr (kBits) tile_bits += s_len8[s & (kWideMaxA - 1)];
                }
                __builtin_nontemporal_store(eo, reinterpret_cast<wf4 *>(mo + i));
                wu2 packed;
                packed[0] = sp[0] | (sp[1] << 16);
                packed[1] = sp[2] | (sp[3] << 16);
                __builtin_nontemporal_store(packed, reinterpret_cast<wu2 *>(su + i));
            }
            add_tile_bits();
            continue;   // workgroup-uniform
        }
        float gv[kWqPer], mv[kWqPer];   // the tile's loads are issued together
#pragma unroll
        for (int k = 0; k < kWqPer; ++k) {
            const uint64_t i = base + (uint64_t)k * kWqThreads + threadIdx.x;
            gv[k] = i < lay.d ? __builtin_nontemporal_load(gu + i) : 0.0f;
            mv[k] = i < lay.d ? mu[i] : 0.0f;
        }
#pragma unroll
        for (int k = 0; k < kWqPer; ++k) {
            const uint64_t i = base + (uint64_t)k * kWqThreads + threadIdx.x;
            if (i >= lay.d) break;
            uint32_t book = tile_book;
            QConst qc = qc0;
            int bias = bias0;
            float gain = gain0, inv_gain = inv_gain0;
            if (!one_layer) {   // workgroup-uniform: the tile crosses into another layer
                uint32_t s_i = seg0;
                while (i >= lay.segs[s_i + 1].offset) ++s_i;   // ends: segs[nseg].offset = d > i
                const uint64_t pair = (uint64_t)u * lay.nseg + s_i;
                bias = lay.bias[pair];
                qc = make_qconst(lay.E, lay.M, bias);
                gain = lay.gain[2 * pair];
                inv_gain = lay.gain[2 * pair + 1];
                book = book_base + (uint32_t)lay.segs[s_i].book;
            }
            const float v = __fadd_rn(gv[k], __fmul_rn(gamma, mv[k]));
            const float y = __fmul_rn(v, gain);
            uint32_t s, flags;
            float q;
            if constexpr (kSR)
                quantize_stochastic(y, qc, lay.E, lay.M, bias, sign_shift, element_random_words(i, u, seed).w[i & 3u], s, q,
                                    flags);
            else quantize(y, qc, sign_shift, s, q, flags);
            q = __fmul_rn(q, inv_gain);
            mo[i] = (flags & 1u) ? 0.0f : __fsub_rn(v, q);
            n_nonfinite += flags & 1u;
            n_clamped += (flags >> 1) & 1u;
            su[i] = (uint16_t)s;
            if (book == cur_book) atomicAdd(&s_hist[s & (kWideMaxA - 1)], 1u);
            else atomicAdd(reinterpret_cast<unsigned long long *>(hist + (uint64_t)book * lay.A + s), 1ull);
            if constexpr (kBits) tile_bits += s_len8[s & (kWideMaxA - 1)];   // (aligned layers: the tile's own table)
        }
        add_tile_bits();
    }
    __syncthreads();
    if (cur_book != 0xffffffffu) flush(cur_book);
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

// One workgroup per table.  A is a power of two (512 .. 4096).  Dynamic LDS: node weights (2 A x 8 bytes),
// parents (2 A x 4 bytes), the leaves' symbols (A x 2 bytes), a round's merged nodes (A x 10 bytes).  Steps: bitonic
// sort of the symbols by (weight, symbol) with the unused ones last; the two-queue merge in rounds of many pairs;
// depth of every leaf; canonical order, the rank of a symbol among those of its length from wavefront ballots
// (wavefront w owns symbols w A/16 .. (w + 1) A/16 - 1, in order).
constexpr int kWbWaves = kWbThreads / 64;
__global__ __launch_bounds__(kWbThreads) void k_build_books_wide(BookWide *__restrict__ books, uint32_t A,
                                                                const uint64_t *__restrict__ weights,
                                                                uint64_t *__restrict__ status)
{
    extern __shared__ uint64_t wb_smem[];
    uint64_t *nw = wb_smem;                                        // [2 A] sorted leaves, then internal nodes
    int *parent = reinterpret_cast<int *>(nw + 2 * (size_t)A);      // [2 A]
    uint16_t *leaf_sym = reinterpret_cast<uint16_t *>(parent + 2 * (size_t)A);   // [A] sorted leaf -> symbol
    uint64_t *tmpw = reinterpret_cast<uint64_t *>(leaf_sym + A);                 // [A] a round's nodes in merged order: weight
    uint16_t *tmpid = reinterpret_cast<uint16_t *>(tmpw + A);                    // [A] and node index
    __shared__ uint32_t cnt[65], off[65];
    __shared__ uint64_t first[65];
    __shared__ uint32_t wcnt[kWbWaves][65];   // symbols of each length in a wavefront's range; then running ranks
    __shared__ int err, s_n;
    __shared__ uint32_t s_maxlen;

    BookWide &B = books[blockIdx.x];
    const uint64_t *w = weights + (uint64_t)blockIdx.x * A;
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint64_t kNone = ~0ull;    // an unused symbol in the sort, an exhausted queue in the merge: refused as a weight

    if (t < 65) { cnt[t] = 0; off[t] = 0; first[t] = 0; }
    for (uint32_t i = t; i < (uint32_t)kWbWaves * 65u; i += kWbThreads) wcnt[i / 65u][i % 65u] = 0;
    if (t == 0) { err = 0; s_maxlen = 0; s_n = 0; }
    for (uint32_t i = t; i < 2 * A; i += kWbThreads) parent[i] = -1;
    __syncthreads();
    int active = 0;
    for (uint32_t s = t; s < A; s += kWbThreads) {
        const uint64_t ws = w[s];
        if (ws == kNone) err = 1;
        active += ws > 0 ? 1 : 0;
        nw[s] = ws ? ws : kNone;
        leaf_sym[s] = (uint16_t)s;
        B.len[s] = 0;
        B.code[s] = 0;
    }
    if (active) atomicAdd(&s_n, active);
    __syncthreads();
    const int nact = s_n;            // number of symbols with a weight

    // ascending (weight, symbol); the keys are distinct, so the order does not depend on the network
    for (uint32_t k = 2; k <= A; k <<= 1) {
        for (uint32_t j = k >> 1; j > 0; j >>= 1) {
            for (uint32_t i = t; i < A; i += kWbThreads) {
                const uint32_t p = i ^ j;
                if (p > i) {
                    const uint64_t wi = nw[i], wp = nw[p];
                    const uint16_t si = leaf_sym[i], sp = leaf_sym[p];
                    const bool gt = wi > wp || (wi == wp && si > sp);
                    if (gt == ((i & k) == 0)) { nw[i] = wp; nw[p] = wi; leaf_sym[i] = sp; leaf_sym[p] = si; }
                }
            }
            __syncthreads();
        }
    }

    // The two-queue merge in rounds.  With T the sum of the two lightest nodes alive, every internal node alive and
    // every leaf of weight <= T is taken before any node created from now on (their weights are >= T; on equal
    // weights a leaf goes before an internal node and an older internal node before a newer one).  So the merged
    // order of those nodes — a leaf's rank is its own index plus the number of lighter internal nodes, an internal
    // node's its own plus the number of leaves that are not heavier — pairs off two by two exactly as the serial
    // merge would; an odd one out stays at the head of its queue.  Every thread keeps the queue positions itself.
    {
        int li = 0, ii = nact, made = nact;   // next leaf, next internal node, next node to create
        auto lower_bound = [&](int lo, int hi, uint64_t x) {   // first index in [lo, hi) with nw[index] >= x
            while (lo < hi) { const int mid = (lo + hi) >> 1; if (nw[mid] < x) lo = mid + 1; else hi = mid; }
            return lo;
        };
        auto upper_bound = [&](int lo, int hi, uint64_t x) {   // first index in [lo, hi) with nw[index] > x
            while (lo < hi) { const int mid = (lo + hi) >> 1; if (nw[mid] <= x) lo = mid + 1; else hi = mid; }
            return lo;
        };
        while (nact >= 2 && !err && (nact - li) + (made - ii) > 1) {   // the same in every thread
            uint64_t c[4] = {li < nact ? nw[li] : kNone, li + 1 < nact ? nw[li + 1] : kNone,
                             ii < made ? nw[ii] : kNone, ii + 1 < made ? nw[ii + 1] : kNone};
            // the two lightest of two sorted pairs
            const uint64_t m1 = c[0] < c[2] ? c[0] : c[2];
            const uint64_t r1 = c[0] < c[2] ? c[1] : c[0], r2 = c[0] < c[2] ? c[2] : c[3];
            const uint64_t m2 = r1 < r2 ? r1 : r2;
            const uint64_t T = m1 + m2;
            if (T < m2 || T == kNone) {   // the table's weights sum to 2^64 - 1 or more
                if (t == 0) err = 1;
                break;
            }
            const int lj = upper_bound(li, nact, T);
            const int bL = lj - li, bI = made - ii, nb = bL + bI;   // nb >= 2: the two lightest are among them
            for (int e = (int)t; e < nb; e += kWbThreads) {
                int node, r;
                if (e < bL) {
                    node = li + e;
                    r = e + (lower_bound(ii, made, nw[node]) - ii);
                } else {
                    node = ii + (e - bL);
                    r = (e - bL) + (upper_bound(li, lj, nw[node]) - li);
                }
                tmpw[r] = nw[node];
                tmpid[r] = (uint16_t)node;
            }
            __syncthreads();
            const int npair = nb >> 1;
            for (int k = (int)t; k < npair; k += kWbThreads) {
                const uint64_t wa = tmpw[2 * k], wb = tmpw[2 * k + 1];
                const uint64_t sum = wa + wb;
                if (sum < wb || sum == kNone) err = 1;
                nw[made + k] = sum;
                parent[tmpid[2 * k]] = made + k;
                parent[tmpid[2 * k + 1]] = made + k;
            }
            __syncthreads();
            int next_li = lj, next_ii = made;
            if (nb & 1) {   // the heaviest of the batch stays: the last internal node unless a leaf is heavier
                if (bI > 0 && (bL == 0 || nw[made - 1] >= nw[lj - 1])) next_ii = made - 1;
                else next_li = lj - 1;
            }
            li = next_li;
            ii = next_ii;
            made += npair;
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

    // lengths present in each wavefront's range of symbols, sub-block of 64 by sub-block
    const uint32_t per_wave = A / kWbWaves;   // 32 .. 256
    auto for_each_length_group = [&](uint32_t myL, auto &&body) {   // body(length, lanes with it), once per length
        uint64_t todo = __ballot(myL != 0u);
        while (todo) {
            const int leader = __ffsll((long long)todo) - 1;
            const uint32_t L0 = (uint32_t)__shfl((int)myL, leader, 64);
            const uint64_t mask = __ballot(myL == L0);
            body(L0, mask);
            todo &= ~mask;
        }
    };
    for (uint32_t sb = 0; sb < per_wave; sb += 64) {
        const uint32_t i = sb + lane;
        const uint32_t myL = i < per_wave ? (uint32_t)B.len[wave * per_wave + i] : 0u;
        for_each_length_group(myL, [&](uint32_t L0, uint64_t mask) {
            if (lane == 0) wcnt[wave][L0] += (uint32_t)__popcll(mask);
        });
    }
    __syncthreads();
    if (t < 65) {   // counts per length; a wavefront's entry becomes the rank of its first symbol of that length
        uint32_t run = 0;
        for (int wv = 0; wv < kWbWaves; ++wv) { const uint32_t c = wcnt[wv][t]; wcnt[wv][t] = run; run += c; }
        cnt[t] = run;
        if (run && t) atomicMax(&s_maxlen, t);
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
    for (uint32_t sb = 0; sb < per_wave; sb += 64) {
        const uint32_t i = sb + lane;
        const uint32_t s_i = wave * per_wave + i;
        const uint32_t myL = i < per_wave ? (uint32_t)B.len[s_i] : 0u;
        for_each_length_group(myL, [&](uint32_t L0, uint64_t mask) {
            const uint32_t base = wcnt[wave][L0];
            if (myL == L0) {
                const uint32_t rank = base + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
                B.code[s_i] = first[L0] + rank;
                B.sorted[off[L0] + rank] = (uint16_t)s_i;
            }
            w_wave_sync_lds();   // every lane has read the base
            if (lane == 0) wcnt[wave][L0] = base + (uint32_t)__popcll(mask);
            w_wave_sync_lds();
        });
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
                e = ((uint32_t)l << 12) | B.sorted[off[l] + (c - f)];
                break;
            }
        }
        B.dec[idx] = (uint16_t)e;
    }
    // second-level tables under the first prefixes that hold only longer codes
    uint32_t long_prefix0 = 1u << kWideDecBits;
    for (int l = kWideDecBits + 1; l <= 64; ++l) {
        if (cnt[l]) { long_prefix0 = (uint32_t)(first[l] >> (l - kWideDecBits)); break; }
    }
    if (t == 0) B.long_prefix0 = long_prefix0;
    for (uint32_t idx = t; idx < (uint32_t)(kWideDec2Tables << kWideDec2Bits); idx += kWbThreads) {
        const uint32_t prefix = long_prefix0 + (idx >> kWideDec2Bits);
        const uint32_t wide = (prefix << kWideDec2Bits) | (idx & ((1u << kWideDec2Bits) - 1u));   // 17 bits
        uint32_t e = 0;
        if (prefix < (1u << kWideDecBits)) {
            for (int l = kWideDecBits + 1; l <= kWideDecBits + kWideDec2Bits; ++l) {
                const uint32_t c = wide >> (kWideDecBits + kWideDec2Bits - l);
                const uint32_t f = (uint32_t)first[l];   // first[l] <= 2^l: in 32 bits
                if (cnt[l] && c >= f && c - f < cnt[l]) {
                    e = ((uint32_t)(l - kWideDecBits) << 12) | B.sorted[off[l] + (c - f)];
                    break;
                }
            }
        }
        B.dec2[idx] = (uint16_t)e;
    }
}

// ---- user side, steps 2 and 3 -------------------------------------------------------------------------------

// Both chunk kernels give a workgroup kWChunksPerWg consecutive chunks of one user (wavefront w takes chunks
// w, w + kWWaves, ...) and keep the code table of the workgroup's first chunk in LDS; a chunk of another table
// (a layer boundary inside the workgroup's range) reads its table from global memory instead.
constexpr int kWChunksPerWave = 4;
constexpr int kWChunksPerWg = kWWaves * kWChunksPerWave;
constexpr uint32_t kWFastCodeBits = 25;   // s_fast entry: length << 25 | codeword, for lengths up to 25
constexpr int kWSymLoads = (kChunk / 2 + 1 + 63) / 64;    // dword loads per lane to cover a chunk at any 2-byte offset (33)
constexpr uint32_t kWSymMask2 = (uint32_t)(kWideMaxA - 1) * 0x10001u;
// A wavefront's LDS words in the coder: 64 rows of 32 + 1 words and one word more.  They hold the staged symbols,
// then (symbols in registers) every lane's own codewords, then the chunk's words; the plain loops for long codes
// keep the symbols in the rows and use a small window behind them.
constexpr int kWRowWords = kWSymRow / 2 - 1;                      // 32
constexpr int kWRowStride = kWRowWords + 1;                       // odd: no bank conflicts
constexpr int kWRegion = kSubsPerChunk * kWRowStride + 1;         // 2113
constexpr int kWWinSlow = 128;
constexpr int kWWinMedium = 2048;                                // the rows' storage as a window
constexpr int kWPackWaveWords = kWRegion + kWWinSlow + 1;
constexpr uint32_t kWFastSlow = 127;                              // length field of a symbol the unrolled coder cannot take
constexpr size_t kWPackLds = sizeof(uint32_t) * (kWideMaxA + kWWaves * kWPackWaveWords);   // 52 KB: three workgroups per CU

// Step 1 of the coder: every lane concatenates the codewords of its 64 symbols (two per word of sym) from bit 0
// of its row, without knowing where they will land in the chunk; its bit count falls out at the end.  A
// codeword enters a 64-bit shift register; it completes at most one 32-bit word, which is stored without a
// branch (a store of the word still being filled is harmless: the slot is written again; stores beyond the row
// go to the row's spare slot).  A lane that met a kWFastSlow entry (a code of more than kWFastCodeBits bits, or
// a symbol without one: a handful of elements in a round of a large vector) codes its row again by itself in a
// rolled loop, its symbols parked in `scratch` (32 words), those entries taken from the table in device memory
// and appended in pieces; nocode counts its symbols without a code.  Returns, for the whole wavefront: kRowsOk;
// kRowsOverflow if a lane's codewords do not fit its row (bits is still every lane's bit count, and no lane met
// a kWFastSlow entry); kRowsSlow if more than kWRedoLanes lanes met one, or one did and a row overflowed.
enum { kRowsOk = 0, kRowsOverflow = 1, kRowsSlow = 2 };
constexpr int kWRedoLanes = 4;
template <bool kFull>
__device__ inline int w_pack_rows(const uint32_t (&sym)[kSub / 2], int cnt, const uint32_t *fast, const BookWide &book,
                                  uint32_t *region, uint32_t *scratch, uint32_t lane, uint32_t &bits, uint32_t &nocode)
{
    uint64_t acc = 0;
    uint32_t np = 0;                                     // bits of acc not yet stored: < 32 between symbols
    const uint32_t row0 = lane * kWRowStride;
    uint32_t waddr = row0;
    const uint32_t wend = row0 + kWRowWords;
    bool left = false;
#pragma unroll
    for (int j = 0; j < kSub; ++j) {
        uint32_t e = fast[(j & 1) ? sym[j >> 1] >> 16 : sym[j >> 1] & 0xffffu];
        if (!kFull) e = (j < cnt) ? e : 0u;              // nothing to append beyond the chunk's end
        const uint32_t L = e >> kWFastCodeBits;          // <= kWFastCodeBits, or kWFastSlow
        np += L;
        left = left || np > 63u;                         // exactly the kWFastSlow entries
        acc = (acc << (L & 63u)) | (e & ((1u << kWFastCodeBits) - 1u));
        const uint32_t rest = np & 31u;
        region[waddr < wend ? waddr : wend] = (uint32_t)(acc >> rest);
        waddr += (np >> 5) & 1u;
        np = rest;
    }
    nocode = 0;
    const uint64_t slow_lanes = __ballot(left);
    if (slow_lanes) {
        if (__popcll(slow_lanes) > kWRedoLanes) return kRowsSlow;
        for (uint64_t todo = slow_lanes; todo; todo &= todo - 1) {   // the same in every lane
            const uint32_t l = (uint32_t)__ffsll((long long)todo) - 1u;
            w_wave_sync_lds();                                       // the scratch words are free
            if (lane == l) {
#pragma unroll
                for (int jj = 0; jj < kSub / 2; ++jj) scratch[jj] = sym[jj];
            }
            w_wave_sync_lds();
            if (lane == l) {
                const uint16_t *mine = reinterpret_cast<const uint16_t *>(scratch);
                acc = 0; np = 0; waddr = row0;
                for (int j = 0; j < (kFull ? kSub : cnt); ++j) {
                    const uint32_t sj = mine[j];
                    const uint32_t e = fast[sj];
                    uint32_t L = e >> kWFastCodeBits;
                    uint64_t code = e & ((1u << kWFastCodeBits) - 1u);
                    if (L == kWFastSlow) {
                        L = book.len[sj];
                        code = book.code[sj];
                        nocode += L == 0u ? 1u : 0u;
                    }
                    while (L) {   // the codeword's leading bits first, at most kWFastCodeBits at a time
                        const uint32_t piece = L < kWFastCodeBits ? L : kWFastCodeBits;
                        L -= piece;
                        np += piece;
                        acc = (acc << piece) | ((code >> L) & ((1ull << piece) - 1ull));
                        const uint32_t rest = np & 31u;
                        region[waddr < wend ? waddr : wend] = (uint32_t)(acc >> rest);
                        waddr += (np >> 5) & 1u;
                        np = rest;
                    }
                }
            }
        }
    }
    const uint32_t whole = waddr - row0;                 // complete words, counted also beyond the row
    if (np) region[waddr < wend ? waddr : wend] = (uint32_t)(acc << (32u - np));
    bits = whole * 32u + np;
    if (__any(whole + (np ? 1u : 0u) > (uint32_t)kWRowWords)) return slow_lanes ? kRowsSlow : kRowsOverflow;
    return kRowsOk;
}

// Step 2: every lane's row holds its `bits` bits; excl: bits of the lanes before it.  The rows go to registers,
// their storage is cleared and becomes the chunk's words: every lane ORs its words in, shifted by its offset.
// On return region[0 .. nwords) holds them, nwords = ceil(sum of bits / 32) <= 64 x 32.
__device__ inline void w_rows_to_window(uint32_t *region, uint32_t lane, uint32_t bits, uint32_t excl, uint32_t nwords)
{
    const uint32_t nw = (bits + 31u) >> 5;               // <= kWRowWords
    uint32_t maxnw = nw;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { const uint32_t y = (uint32_t)__shfl_xor((int)maxnw, o, 64); maxnw = maxnw > y ? maxnw : y; }
    uint32_t r[kWRowWords];
    const uint32_t *row = region + lane * kWRowStride;
#pragma unroll
    for (int i = 0; i < kWRowWords; ++i) {
        r[i] = 0u;
        if ((uint32_t)i < maxnw) r[i] = (uint32_t)i < nw ? row[i] : 0u;
    }
    w_wave_sync_lds();                                   // all rows are in registers
    for (uint32_t i = lane; i <= nwords; i += 64) region[i] = 0u;
    w_wave_sync_lds();
    const uint32_t sh = excl & 31u, w0 = excl >> 5;
    uint32_t prev = 0u;
#pragma unroll
    for (int i = 0; i < kWRowWords; ++i) {
        if ((uint32_t)i < maxnw) {
            const uint32_t out = __builtin_amdgcn_alignbit(prev, r[i], sh);   // ({prev, r[i]} >> sh), low word
            if (out) atomicOr(&region[w0 + (uint32_t)i], out);
            prev = r[i];
        }
    }
    const uint32_t tail = __builtin_amdgcn_alignbit(prev, 0u, sh);   // what the shift pushed out of the last word
    if (sh && tail && nw) atomicOr(&region[w0 + nw], tail);
    w_wave_sync_lds();
}

__global__ __launch_bounds__(kWThreads) void k_chunk_bits_wide(Layout lay, const uint16_t *__restrict__ sym,
                                                              uint64_t sym_stride, const BookWide *__restrict__ books,
                                                              uint32_t *__restrict__ chunk_bits)
{
    __shared__ uint8_t s_len[kWideMaxA];
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t c_base = (uint64_t)blockIdx.x * kWChunksPerWg;   // < nchunks by the grid
    const uint32_t u = blockIdx.y;
    const uint32_t wg_book = w_chunk(lay, c_base, u).book;
    for (uint32_t i = threadIdx.x; i < (uint32_t)kWideMaxA; i += kWThreads)
        s_len[i] = i < lay.A ? books[wg_book].len[i] : (uint8_t)0;
    __syncthreads();
    for (int it = 0; it < kWChunksPerWave; ++it) {
        const uint64_t c = c_base + (uint64_t)it * kWWaves + wave;
        if (c >= lay.nchunks) break;   // whole wavefront; no workgroup barriers below
        const WChunk k = w_chunk(lay, c, u);
        const uint16_t *src = sym + (uint64_t)u * sym_stride + k.e0;
        uint32_t total = 0;
        if (k.book == wg_book) {
            uint32_t done = 0;
            if ((reinterpret_cast<uintptr_t>(src) & 15u) == 0) {   // eight symbols per load
                const uint4 *src8 = reinterpret_cast<const uint4 *>(src);
                uint4 v[kChunk / 8 / 64];   // a whole chunk is eight loads per lane, all requested before the first is used
#pragma unroll
                for (int r = 0; r < kChunk / 8 / 64; ++r) {
                    const uint32_t i = lane + 64u * r;
                    v[r] = i < (k.n >> 3) ? src8[i] : make_uint4(0u, 0u, 0u, 0u);
                }
#pragma unroll
                for (int r = 0; r < kChunk / 8 / 64; ++r) {
                    if (lane + 64u * r >= (k.n >> 3)) continue;
                    const uint32_t w[4] = {v[r].x, v[r].y, v[r].z, v[r].w};
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        total += (uint32_t)s_len[w[q] & (kWideMaxA - 1)] + (uint32_t)s_len[(w[q] >> 16) & (kWideMaxA - 1)];
                }
                done = k.n & ~7u;
            }
            for (uint32_t e = done + lane; e < k.n; e += 64) total += s_len[src[e] & (kWideMaxA - 1)];
        } else {
            const uint8_t *len = books[k.book].len;
            for (uint32_t e = lane; e < k.n; e += 64) total += len[src[e] & (kWideMaxA - 1)];
        }
        total = w_wave_sum(total);
        if (lane == 0) chunk_bits[(uint64_t)u * lay.nchunks + c] = total;
    }
}

__global__ __launch_bounds__(kWThreads, 3) void k_pack_wide(Layout lay, const uint16_t *__restrict__ sym, uint64_t sym_stride,
                                                        const BookWide *__restrict__ books,
                                                        const uint64_t *__restrict__ chunk_offset,
                                                        uint16_t *__restrict__ sub_bits, uint32_t *__restrict__ words,
                                                        uint64_t words_stride, uint64_t *__restrict__ status)
{
    extern __shared__ uint32_t wp_smem[];   // kWPackLds bytes
    uint32_t *s_fast = wp_smem;                      // [kWideMaxA]
    uint32_t *s_wave_all = s_fast + kWideMaxA;       // [kWWaves][kWPackWaveWords]
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t c_base = (uint64_t)blockIdx.x * kWChunksPerWg;   // < nchunks by the grid
    const uint32_t u = blockIdx.y;
    const uint32_t wg_book = w_chunk(lay, c_base, u).book;
    {
        const BookWide &tb = books[wg_book];
        uint32_t tl[kWideMaxA / kWThreads], tc[kWideMaxA / kWThreads];   // the loads are issued together
#pragma unroll
        for (int r = 0; r < kWideMaxA / kWThreads; ++r) {
            const uint32_t i = threadIdx.x + (uint32_t)r * kWThreads;
            tl[r] = i < lay.A ? (uint32_t)tb.len[i] : 0u;
            tc[r] = i < lay.A ? (uint32_t)tb.code[i] : 0u;
        }
#pragma unroll
        for (int r = 0; r < kWideMaxA / kWThreads; ++r) {
            const uint32_t i = threadIdx.x + (uint32_t)r * kWThreads;
            // no code, or a longer one than an entry holds: kWFastSlow
            s_fast[i] = (tl[r] >= 1u && tl[r] <= kWFastCodeBits) ? ((tl[r] << kWFastCodeBits) | tc[r]) : (kWFastSlow << kWFastCodeBits);
        }
    }
    __syncthreads();
    uint32_t *region = s_wave_all + wave * kWPackWaveWords;
    for (int it = 0; it < kWChunksPerWave; ++it) {
        const uint64_t c = c_base + (uint64_t)it * kWWaves + wave;
        if (c >= lay.nchunks) break;   // whole wavefront; wavefront-level synchronisation only below
        const WChunk k = w_chunk(lay, c, u);
        const BookWide &book = books[k.book];
        const uint16_t *src = sym + (uint64_t)u * sym_stride + k.e0;
        // The chunk's symbols, at any 2-byte offset and of any length: coalesced dwords from the 4-byte boundary
        // below the chunk go to LDS rows of 32 + 1 words (word i of the chunk at i + i / 32), from which lane l
        // funnels its 64 symbols (words 32 l .. 32 l + 32) into registers, two per word.
        const uint32_t shift = (uint32_t)(reinterpret_cast<uintptr_t>(src) >> 1) & 1u;
        const uint32_t *src32 = reinterpret_cast<const uint32_t *>(src - shift);
        const uint32_t ndw = (shift + k.n + 1u) >> 1;      // <= kChunk / 2 + 1
        uint32_t tmp[kWSymLoads];
#pragma unroll
        for (int r = 0; r < kWSymLoads; ++r) {
            const uint32_t i = lane + 64u * r;
            tmp[r] = i < ndw ? __builtin_nontemporal_load(src32 + i) : 0u;   // all requested before the first is used
        }
        const uint64_t off = chunk_offset[(uint64_t)u * (lay.nchunks + 1) + c];
        w_wave_sync_lds();   // the previous chunk's words have been copied out
#pragma unroll
        for (int r = 0; r < kWSymLoads; ++r) {
            const uint32_t i = lane + 64u * r;
            if (i < (uint32_t)kChunk / 2 + 1) region[i + (i >> 5)] = tmp[r];   // word 2048 lands at 2112
        }
        w_wave_sync_lds();
        const int first = (int)lane * kSub;
        const int cnt = (int)k.n - first < 0 ? 0 : ((int)k.n - first > kSub ? kSub : (int)k.n - first);
        uint32_t *row32 = region + lane * kWRowStride;
        uint32_t symw[kSub / 2];
        {
            uint32_t cur = row32[0];
#pragma unroll
            for (int jj = 0; jj < kSub / 2; ++jj) {
                const uint32_t nxt = row32[jj + 1 + (jj == kSub / 2 - 1 ? 1 : 0)];   // row32[32] is the row's spare slot
                symw[jj] = (shift ? __builtin_amdgcn_alignbit(nxt, cur, 16u) : cur) & kWSymMask2;   // table indices stay below kWideMaxA
                cur = nxt;
            }
        }
        w_wave_sync_lds();   // every lane holds its symbols: the rows are free

        uint32_t bits = 0;
        const bool in_lds = k.book == wg_book;   // whole wavefront: the table in LDS is this chunk's
        int rows = kRowsSlow;
        if (in_lds) {
            uint32_t nocode = 0;
            rows = k.n == (uint32_t)kChunk
                       ? w_pack_rows<true>(symw, cnt, s_fast, book, region, region + kWRegion, lane, bits, nocode)
                       : w_pack_rows<false>(symw, cnt, s_fast, book, region, region + kWRegion, lane, bits, nocode);
            if (rows != kRowsSlow && nocode)   // (the plain loops below count them themselves)
                atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_NOCODE), (unsigned long long)nocode);
        }
        const bool fast_ok = rows == kRowsOk;
        const uint16_t *row = reinterpret_cast<const uint16_t *>(row32);
        // what the plain loops know of a symbol: from the table in LDS where that is this chunk's and holds the
        // symbol's code, else from device memory
        auto lookup = [&](uint32_t sj, uint32_t &L, uint64_t &code) {
            const uint32_t e = in_lds ? s_fast[sj] : (kWFastSlow << kWFastCodeBits);
            L = e >> kWFastCodeBits;
            code = e & ((1u << kWFastCodeBits) - 1u);
            if (L == kWFastSlow) { L = book.len[sj]; code = book.code[sj]; }
        };
        if (rows == kRowsSlow) {
            // a long code, a symbol without one, or another table: the symbols go back to the rows, plain loops
            w_wave_sync_lds();
#pragma unroll
            for (int jj = 0; jj < kSub / 2; ++jj) row32[jj] = symw[jj];
            w_wave_sync_lds();
            uint32_t nocode = 0;
            bits = 0;
            for (int j = 0; j < cnt; ++j) {
                uint32_t L;
                uint64_t code;
                lookup(row[j], L, code);
                nocode += L == 0u ? 1u : 0u;
                bits += L;
            }
            if (nocode)
                atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_NOCODE), (unsigned long long)nocode);
        }
        sub_bits[((uint64_t)u * lay.nchunks + c) * kSubsPerChunk + lane] = (uint16_t)bits;
        const uint32_t incl = w_wave_inclusive_scan(bits, lane);
        const uint32_t excl = incl - bits;
        const uint32_t chunk_total = __shfl(incl, 63, 64);
        const uint32_t nwords = (chunk_total + 31u) >> 5;
        const uint64_t off_words = off >> 5;
        if (off_words + nwords > words_stride) {   // whole wavefront
            if (lane == 0) atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CAPACITY), 1ull);
            continue;
        }
        uint32_t *dst = words + (uint64_t)u * words_stride + off_words;
        if (fast_ok) {
            w_rows_to_window(region, lane, bits, excl, nwords);
            for (uint32_t i = lane; i < nwords; i += 64) __builtin_nontemporal_store(region[i], dst + i);
            continue;
        }
        // Rows too short for some lane (more than 16 bits per symbol on average): the codewords are appended at
        // their final bit offsets instead, entries from the table in LDS, the rows' storage as the window.  After
        // the plain loops above: the same from the rows' symbols, a small window behind them.
        const bool medium = rows == kRowsOverflow;
        uint32_t *win = medium ? region : region + kWRegion;
        const uint32_t wcap = medium ? (uint32_t)kWWinMedium : (uint32_t)kWWinSlow;
        for (uint32_t wbase = 0; wbase < nwords; wbase += wcap) {
            const uint32_t wn = nwords - wbase < wcap ? nwords - wbase : wcap;
            w_wave_sync_lds();
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
            // a lane whose bits all lie outside this window has nothing to add
            const bool overlaps = excl + bits > wbase * 32u && excl < (wbase + wn) * 32u;
            if (medium) {   // whole wavefront; every existing symbol has a code of at most kWFastCodeBits bits
#pragma unroll
                for (int j = 0; j < kSub; ++j) {
                    const uint32_t e = s_fast[(j & 1) ? symw[j >> 1] >> 16 : symw[j >> 1] & 0xffffu];
                    if (overlaps && j < cnt) append(e & ((1u << kWFastCodeBits) - 1u), e >> kWFastCodeBits);
                }
            }
            for (int j = 0; !medium && overlaps && j < cnt; ++j) {
                uint32_t L;
                uint64_t code;
                lookup(row[j], L, code);
                if (!L) continue;
                if (L > 32u) {
                    append(code >> 32, L - 32u);
                    code &= 0xffffffffull;
                    L = 32u;
                }
                append(code, L);
            }
            if (overlaps && np && wi < wn) atomicOr(&win[wi], (uint32_t)(acc << (32u - np)));
            w_wave_sync_lds();
            for (uint32_t i = lane; i < wn; i += 64) dst[wbase + i] = win[i];
            w_wave_sync_lds();
        }
    }
}

// ---- PS side ----------------------------------------------------------------------------------------------

// What the decoder keeps in LDS of one table; the symbols in canonical order, which only the search for a code
// that neither table holds needs, stay in device memory.  The second-level tables come last: a wavefront that
// keeps a table of its own (a set of tables per user) leaves them out - kWTabsShort bytes per table, so that
// twice as many wavefronts fit a CU - and finds every code of more than kWideDecBits bits by value.
struct WideTabs {
    uint16_t dec[1 << kWideDecBits];
    uint64_t first[65];
    uint64_t upper[65];    // (first[L] + count[L]) left-aligned in 64 bits: every code of L or fewer bits lies below
    uint32_t count[65];
    uint32_t offset[65];
    uint32_t maxlen;
    uint32_t long_prefix0;
    uint16_t dec2[kWideDec2Tables << kWideDec2Bits];
};
constexpr size_t kWTabsShort = offsetof(WideTabs, dec2);
static_assert(kWTabsShort % 8 == 0 && sizeof(WideTabs) % 8 == 0, "tables follow each other in LDS");

template <bool kDec2>
__device__ inline void w_load_tabs(WideTabs *T, const BookWide &book, uint32_t t, uint32_t nthreads)
{
    const uint32_t *src = reinterpret_cast<const uint32_t *>(book.dec);   // two entries per word
    uint32_t *dst = reinterpret_cast<uint32_t *>(T->dec);
#pragma unroll 8
    for (uint32_t i = t; i < (1u << kWideDecBits) / 2; i += nthreads) dst[i] = src[i];
    if constexpr (kDec2) {
        src = reinterpret_cast<const uint32_t *>(book.dec2);
        dst = reinterpret_cast<uint32_t *>(T->dec2);
#pragma unroll 8
        for (uint32_t i = t; i < (uint32_t)(kWideDec2Tables << kWideDec2Bits) / 2; i += nthreads) dst[i] = src[i];
    }
#pragma unroll 1
    for (uint32_t i = t; i < 65u; i += nthreads) {
        const uint64_t f = book.first[i];
        const uint32_t c = book.count[i];
        T->first[i] = f;
        T->count[i] = c;
        T->offset[i] = book.offset[i];
        uint64_t up = ~0ull;   // lengths 0 and 64, and sums that leave L bits, bound nothing
        if (i >= 1u && i < 64u && ((f + c) >> i) == 0) up = (f + c) << (64u - i);
        T->upper[i] = up;
    }
    if (t == 0) { T->maxlen = book.maxlen > 64u ? 64u : book.maxlen; T->long_prefix0 = book.long_prefix0; }
}

// A chunk's payload words in global memory; reads nothing outside w[0 .. nw).
struct WGlobalWords {
    const uint32_t *w;
    uint32_t nw;
    __device__ inline uint32_t word(uint32_t i) const { return i < nw ? w[i] : 0u; }
};

// The three words of a chunk's payload at the read position, and the one after them, which is requested when the
// position enters a new word and first used when it enters the next one: the load has the symbols in between
// to complete.
template <class Src>
struct WReader {
    Src src;
    uint32_t i0, w0, w1, w2, w3;
    __device__ inline void seek(uint32_t pos)
    {
        i0 = pos >> 5;
        w0 = src.word(i0);
        w1 = src.word(i0 + 1u);
        w2 = src.word(i0 + 2u);
        w3 = src.word(i0 + 3u);
    }
    // the 32 bits from bit `pos` on; pos never decreases between calls
    __device__ inline uint32_t window32(uint32_t pos)
    {
        const uint32_t i = pos >> 5, s0 = pos & 31u;
        if (i == i0 + 1u) { w0 = w1; w1 = w2; w2 = w3; w3 = src.word(i + 3u); i0 = i; }
        else if (i != i0) seek(pos);
        return s0 ? __builtin_amdgcn_alignbit(w0, w1, 32u - s0) : w0;   // ({w0, w1} >> (32 - s0)), low word
    }
    // the 32 bits after those, for the same pos
    __device__ inline uint32_t next32(uint32_t pos) const
    {
        const uint32_t s0 = pos & 31u;
        return s0 ? __builtin_amdgcn_alignbit(w1, w2, 32u - s0) : w1;
    }
};

constexpr int kWUpRegs = 12;   // lengths kWideDecBits + 1 .. kWideDecBits + 12 have their bound in a register

// The bounds of lengths kWideDecBits + 1 .. kWideDecBits + kWUpRegs, top 32 bits (exact: a bound of length
// l <= 32 has no lower bits); lengths from maxlen on bound nothing.
struct WUpper32 {
    uint32_t up[kWUpRegs];
    __device__ inline void load(const WideTabs *T)
    {
#pragma unroll
        for (int t = 0; t < kWUpRegs; ++t) {
            const uint32_t l = kWideDecBits + 1 + t;
            up[t] = l < T->maxlen ? (uint32_t)(T->upper[l] >> 32) : 0xffffffffu;
        }
    }
};

template <bool kDec2, class Src>
__device__ inline uint32_t w_decode_one(WReader<Src> &r, uint32_t pos, const WideTabs *T, const uint16_t *__restrict__ sorted,
                                        const WUpper32 &U32, uint32_t &len)
{
    const uint32_t hi = r.window32(pos);
    const uint32_t prefix = hi >> (32 - kWideDecBits);
    const uint32_t e = T->dec[prefix];
    if (e) { len = e >> 12; return e & 0xfffu; }
    if constexpr (kDec2) {
        const uint32_t tab = prefix - T->long_prefix0;   // wraps below it: no table
        if (tab < (uint32_t)kWideDec2Tables) {
            const uint32_t e2 = T->dec2[(tab << kWideDec2Bits) | ((hi >> (32 - kWideDecBits - kWideDec2Bits)) & ((1u << kWideDec2Bits) - 1u))];
            if (e2) { len = kWideDecBits + (e2 >> 12); return e2 & 0xfffu; }
        }
    }
    const uint32_t maxlen = T->maxlen;   // <= 64
    len = 0;
    if (maxlen <= (uint32_t)kWideDecBits) return 0u;   // every code is in the prefix table
    // the bounds in two halves: few codes reach the second
    uint32_t L = kWideDecBits + 1;
#pragma unroll
    for (int t = 0; t < kWUpRegs / 2; ++t) L += hi >= U32.up[t] ? 1u : 0u;
    if (L == kWideDecBits + 1 + kWUpRegs / 2) {
#pragma unroll
        for (int t = kWUpRegs / 2; t < kWUpRegs; ++t) L += hi >= U32.up[t] ? 1u : 0u;
    }
    uint64_t full = 0;
    if (L == kWideDecBits + 1 + kWUpRegs) {   // longer than the registers cover
        full = ((uint64_t)hi << 32) | r.next32(pos);
        for (uint32_t l = L; l < maxlen; ++l) L += full >= T->upper[l] ? 1u : 0u;
    }
    L = min(L, maxlen);   // a window of ones passes the bounds that bound nothing, too
    uint32_t rank;
    if (L <= 32u) {       // first[L] < 2^L: its low word is all of it
        const uint32_t cde = hi >> (32u - L);
        const uint32_t f = (uint32_t)T->first[L];
        if (cde < f) return 0u;
        rank = cde - f;
    } else {
        if (!full) full = ((uint64_t)hi << 32) | r.next32(pos);
        const uint64_t cde = full >> (64u - L);
        const uint64_t f = T->first[L];
        if (cde < f || cde - f >= (uint64_t)kWideMaxA) return 0u;
        rank = (uint32_t)(cde - f);
    }
    if (rank >= T->count[L]) return 0u;
    len = L;
    return sorted[(T->offset[L] + rank) & (kWideMaxA - 1)];
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

constexpr int kWDecWaves = 8;          // wavefronts of a decode workgroup with one set of code tables for all users
constexpr int kWDecWavesPerUser = 4;   // and with a set per user (a table per wavefront in LDS)
constexpr int kWDecBlock = 32;         // symbols a lane decodes between two copies to device memory
constexpr int kWDecRow = kWDecBlock + 2;                  // 16-bit units of a lane's row: 17 words, odd
constexpr int kWDecRowsWave = kSubsPerChunk * kWDecRow;   // 16-bit units of a wavefront's 64 rows
static_assert(kSub % kWDecBlock == 0 && (kWDecRowsWave * sizeof(uint16_t)) % 8 == 0, "blocks per sub-chunk, table alignment");

template <bool kPerUser>
__global__ __launch_bounds__(64 * kWDecWaves) void k_decode_wide(Layout lay, const uint32_t *__restrict__ words,
                                                                uint64_t words_stride,
                                                                const uint64_t *__restrict__ chunk_offset,
                                                                const uint16_t *__restrict__ sub_bits,
                                                                const BookWide *__restrict__ books, uint16_t *__restrict__ sym,
                                                                uint64_t sym_stride, float *__restrict__ q, uint64_t q_stride,
                                                                uint64_t *__restrict__ status)
{
    // The wavefronts of a workgroup decode the same chunk of as many users: with one set of code tables for all
    // users they share one copy of the chunk's table, else each keeps its own.  A lane decodes its sub-chunk
    // kWDecBlock symbols at a time into a row of LDS (rows for all 64 symbols would leave room for 12 wavefronts
    // per CU; blocks of 16 for 32, but store 32 bytes at a time); after each block the rows go out in element
    // order, 32 consecutive elements per row and 2 rows per store.
    extern __shared__ uint64_t wd_smem[];
    const uint32_t nthreads = blockDim.x, nwaves = blockDim.x >> 6;
    uint16_t *s_rows = reinterpret_cast<uint16_t *>(wd_smem);                                // [nwaves][64 rows]
    unsigned char *s_tabs = reinterpret_cast<unsigned char *>(s_rows + nwaves * kWDecRowsWave);   // one table, or nwaves short ones
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t c = blockIdx.x;
    const uint32_t u = blockIdx.y * nwaves + wave;
    if (!kPerUser) {
        w_load_tabs<true>(reinterpret_cast<WideTabs *>(s_tabs), books[w_chunk(lay, c, 0).book], threadIdx.x, nthreads);
        __syncthreads();
    }
    if (u >= lay.U) return;  // whole wavefront; wavefront-level synchronisation only below
    const WChunk k = w_chunk(lay, c, u);
    const BookWide &book = books[k.book];
    WideTabs *T = reinterpret_cast<WideTabs *>(s_tabs + (kPerUser ? wave * kWTabsShort : 0u));
    uint16_t *rows = s_rows + wave * kWDecRowsWave;
    const WIndex ix = w_read_index(lay, c, u, words, words_stride, chunk_offset, sub_bits, lane);
    if (kPerUser) w_load_tabs<false>(T, book, lane, 64);
    w_wave_sync_lds();
    WUpper32 U32;
    U32.load(T);
    const uint32_t p0 = w_wave_inclusive_scan(ix.sb, lane) - ix.sb;
    const int first = (int)lane * kSub;
    const int cnt = (int)k.n - first < 0 ? 0 : ((int)k.n - first > kSub ? kSub : (int)k.n - first);
    const uint64_t pair = (uint64_t)u * lay.nseg + k.seg;
    const int bias = lay.bias[pair];
    const float inv_gain = lay.gain[2 * pair + 1];
    uint32_t pos = p0;
    bool bad = false;
    WReader<WGlobalWords> rd{WGlobalWords{ix.w, ix.nw}, 0u, 0u, 0u, 0u, 0u};
    rd.seek(p0);
    const uint32_t col = lane & (uint32_t)(kWDecBlock - 1), rsub = lane / (uint32_t)kWDecBlock;   // of the copy
    for (int blk = 0; blk < kSub / kWDecBlock; ++blk) {
        if ((uint32_t)(blk * kWDecBlock) >= k.n) break;   // wavefront-uniform: no lane has a symbol left
        for (int jj = 0; jj < kWDecBlock; ++jj) {
            if (blk * kWDecBlock + jj < cnt) {
                uint32_t len;
                const uint32_t s = w_decode_one<!kPerUser>(rd, pos, T, book.sorted, U32, len);
                if (len == 0u) { bad = true; len = 1u; }
                pos += len;
                rows[lane * kWDecRow + jj] = (uint16_t)s;
            }
        }
        w_wave_sync_lds();
        for (uint32_t r = rsub; r < (uint32_t)kSubsPerChunk; r += 64u / (uint32_t)kWDecBlock) {
            const uint32_t e = 64u * r + (uint32_t)(blk * kWDecBlock) + col;   // element of the chunk
            if (e < k.n) {
                const uint32_t s = rows[r * kWDecRow + col];
                if (sym) sym[(uint64_t)u * sym_stride + k.e0 + e] = (uint16_t)s;
                if (q) q[(uint64_t)u * q_stride + k.e0 + e] = __fmul_rn(__uint_as_float(symbol_value_bits(s, lay.E, lay.M, bias)), inv_gain);
            }
        }
        w_wave_sync_lds();   // the rows are free again
    }
    if (bad || pos - p0 != ix.sb || !ix.ok)
        atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CORRUPT), 1ull);
}

constexpr int kWAccStride = kSub + 1;
constexpr int kWAccWords = kSubsPerChunk * kWAccStride;
constexpr int kWAggWaves = 8;          // wavefronts of a workgroup with one set of code tables for all users
constexpr int kWAggWavesPerUser = 4;   // and with a set per user (a table per wavefront in LDS)
constexpr int kWAggThreads = 64 * kWAggWaves;

// One workgroup per chunk; wavefront w of n decodes users w, w + n, ... and adds their values to the chunk's fp64
// sums in LDS.  With one set of code tables for all users the workgroup keeps a single copy of the chunk's table,
// else one per wavefront.
template <bool kPerUser>
__global__ __launch_bounds__(kWAggThreads, kPerUser ? 2 : 6) void k_aggregate_wide(Layout lay, const uint32_t *__restrict__ words,
                                                                uint64_t words_stride,
                                                                const uint64_t *__restrict__ chunk_offset,
                                                                const uint16_t *__restrict__ sub_bits,
                                                                const BookWide *__restrict__ books, float *__restrict__ out,
                                                                float *__restrict__ model, float eta,
                                                                uint64_t *__restrict__ status)
{
    extern __shared__ uint64_t wa_smem[];
    double *s_acc = reinterpret_cast<double *>(wa_smem);                      // [64][kWAccStride]
    unsigned char *s_tabs = reinterpret_cast<unsigned char *>(s_acc + kWAccWords);   // one table, or a short one per wavefront
    const uint32_t t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const uint64_t c = blockIdx.x;
    const WChunk k0 = w_chunk(lay, c, 0);
    const uint32_t nthreads = blockDim.x, nwaves = blockDim.x >> 6;
    for (uint32_t i = t; i < (uint32_t)kWAccWords; i += nthreads) s_acc[i] = 0.0;
    if (!kPerUser) w_load_tabs<true>(reinterpret_cast<WideTabs *>(s_tabs), books[k0.book], t, nthreads);
    __syncthreads();
    WideTabs *T = reinterpret_cast<WideTabs *>(s_tabs + (kPerUser ? wave * kWTabsShort : 0u));
    const uint32_t sign_shift = (uint32_t)(lay.E + lay.M), kmask = (1u << sign_shift) - 1u, mshift = 23u - (uint32_t)lay.M;
    WUpper32 U32;
    if (!kPerUser) U32.load(T);
    for (uint32_t u = wave; u < lay.U; u += nwaves) {
        const WChunk k = w_chunk(lay, c, u);
        const BookWide &book = books[k.book];
        const WIndex ix = w_read_index(lay, c, u, words, words_stride, chunk_offset, sub_bits, lane);
        if (kPerUser) {
            w_wave_sync_lds();   // the previous user's table has been read
            w_load_tabs<false>(T, book, lane, 64);
            w_wave_sync_lds();
            U32.load(T);
        }
        const uint32_t p0 = w_wave_inclusive_scan(ix.sb, lane) - ix.sb;
        const int first = (int)lane * kSub;
        const int cnt = (int)k.n - first < 0 ? 0 : ((int)k.n - first > kSub ? kSub : (int)k.n - first);
        const uint64_t pair = (uint64_t)u * lay.nseg + k.seg;
        const int bias = lay.bias[pair];
        const float inv_gain = lay.gain[2 * pair + 1];
        const bool scaled = inv_gain != 1.0f;
        const uint32_t ebias = (uint32_t)(127 - bias) << 23;
        double *acc = s_acc + lane * kWAccStride;
        uint32_t pos = p0;
        bool bad = false;
        WReader<WGlobalWords> rd{WGlobalWords{ix.w, ix.nw}, 0u, 0u, 0u, 0u, 0u};
        rd.seek(p0);
        for (int j = 0; j < cnt; ++j) {
            uint32_t len;
            const uint32_t s = w_decode_one<!kPerUser>(rd, pos, T, book.sorted, U32, len);
            if (len == 0u) { bad = true; len = 1u; }
            pos += len;
            // a representative of a normal binade is the symbol's exponent and mantissa fields moved to their fp32
            // places plus the difference of the biases
            const uint32_t k = s & kmask;
            uint32_t vb = (k << mshift) + ebias;
            if (k < (1u << lay.M)) vb = symbol_value_bits(k, lay.E, lay.M, bias);   // zero and the subnormal row
            vb |= (s >> sign_shift) << 31;
            float val = __uint_as_float(vb);
            if (scaled) val = __fmul_rn(val, inv_gain);   // (the same in every lane)
            __hip_atomic_fetch_add(&acc[j], (double)val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        if (bad || pos - p0 != ix.sb || !ix.ok)
            atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CORRUPT), 1ull);
    }
    __syncthreads();
    const double inv_u = 1.0 / (double)lay.U;
    const double eta64 = (double)eta;
    for (uint32_t e = t; e < k0.n; e += nthreads) {
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
    const size_t lds = (size_t)2 * A * (sizeof(uint64_t) + sizeof(int)) + (size_t)A * (2 * sizeof(uint16_t) + sizeof(uint64_t));   // 144 KB at A = 4096
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
    // a code that is held and layers on the quantizer's tile grid: the chunks' sizes come out of the first sweep
    const bool bits_in_sweep = a.mode == CO3_BOOK_FIXED && lay.tile_aligned && lay.nchunks;
    {
        // the partial counts and, behind them in the workspace, the chunk sizes the sweep adds to
        const uint64_t zero_n = bits_in_sweep ? (w_up256(hist_rep_n * sizeof(uint64_t)) + w_up256((size_t)lay.U * lay.nchunks * sizeof(uint32_t))) / sizeof(uint64_t)
                                              : hist_rep_n;
        ProfScope prof(K_ZERO, s);
        hipLaunchKernelGGL(k_zero_wide, dim3((uint32_t)((zero_n + 255) / 256)), dim3(256), 0, s, hist_rep, zero_n);
    }
    if (lay.d) {
        ProfScope prof(K_QUANTIZE, s);
        const dim3 grid((uint32_t)((lay.d + (uint64_t)kWqTile * kWqTiles - 1) / ((uint64_t)kWqTile * kWqTiles)), lay.U);
        auto launch = [&](auto kernel) {
            hipLaunchKernelGGL(kernel, grid, dim3(kWqThreads), 0, s, lay, a.g, a.m, a.m_out, sym, sym_stride, a.row_stride,
                               a.gamma, a.seed, hist_rep, static_cast<const BookWide *>(books), chunk_bits, a.status);
        };
        if (a.rounding == CO3_ROUND_STOCHASTIC) {
            if (bits_in_sweep) launch(k_quantize_wide<true, true>);
            else launch(k_quantize_wide<true, false>);
        } else {
            if (bits_in_sweep) launch(k_quantize_wide<false, true>);
            else launch(k_quantize_wide<false, false>);
        }
    }
    {
        ProfScope prof(K_REDUCE_HIST, s);
        hipLaunchKernelGGL(k_reduce_hist_wide, dim3((uint32_t)((hist_n + 255) / 256)), dim3(256), 0, s, hist_rep, hist, hist_n);
    }
    if (a.mode == CO3_BOOK_EMPIRICAL) {
        hipError_t e = launch_build_books_wide(books, lay.nbooks, lay.A, hist, a.status, s);
        if (e != hipSuccess) return e;
    }
    const uint32_t gx = (uint32_t)((lay.nchunks + kWChunksPerWg - 1) / kWChunksPerWg);
    if (lay.nchunks && !bits_in_sweep) {
        ProfScope prof(K_CHUNK_BITS, s);
        hipLaunchKernelGGL(k_chunk_bits_wide, dim3(gx, lay.U), dim3(kWThreads), 0, s, lay, sym, sym_stride, books, chunk_bits);
    }
    hipError_t e = launch_scan_chunks(lay, chunk_bits, a.chunk_offset, a.payload_bits, s);   // the byte path's scan
    if (e != hipSuccess) return e;
    if (lay.nchunks) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_pack_wide), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)kWPackLds);
        if (e != hipSuccess) return e;
        ProfScope prof(K_PACK, s);
        hipLaunchKernelGGL(k_pack_wide, dim3(gx, lay.U), dim3(kWThreads), kWPackLds, s, lay, sym, sym_stride, books,
                           a.chunk_offset, a.sub_bits, a.words, a.words_stride, a.status);
    }
    return hipGetLastError();
}

hipError_t launch_decode_wide(const Layout &lay, const co3_decode_args &a, const BookWide *books, hipStream_t s)
{
    if (lay.U == 0 || lay.nchunks == 0) return hipSuccess;
    const uint64_t sym_stride = symbol_row_stride(lay.d);
    const uint32_t nwaves = lay.per_user_books ? kWDecWavesPerUser : kWDecWaves;
    const size_t lds = (size_t)nwaves * kWDecRowsWave * sizeof(uint16_t) +
                       (lay.per_user_books ? (size_t)nwaves * kWTabsShort : sizeof(WideTabs));   // 52 KB, or 55 KB with a set per user
    const void *fn = lay.per_user_books ? reinterpret_cast<const void *>(&k_decode_wide<true>)
                                        : reinterpret_cast<const void *>(&k_decode_wide<false>);
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    ProfScope prof(K_DECODE, s);
    const dim3 grid((uint32_t)lay.nchunks, (lay.U + nwaves - 1) / nwaves);
    if (lay.per_user_books)
        hipLaunchKernelGGL(k_decode_wide<true>, grid, dim3(64 * nwaves), lds, s, lay, a.words, a.words_stride, a.chunk_offset,
                           a.sub_bits, books, reinterpret_cast<uint16_t *>(a.symbols), sym_stride, a.q, a.q_stride, a.status);
    else
        hipLaunchKernelGGL(k_decode_wide<false>, grid, dim3(64 * nwaves), lds, s, lay, a.words, a.words_stride, a.chunk_offset,
                           a.sub_bits, books, reinterpret_cast<uint16_t *>(a.symbols), sym_stride, a.q, a.q_stride, a.status);
    return hipGetLastError();
}

hipError_t launch_aggregate_wide(const Layout &lay, const co3_aggregate_args &a, const BookWide *books, hipStream_t s)
{
    if (lay.U == 0 || lay.nchunks == 0) return hipSuccess;
    const uint32_t nwaves = lay.per_user_books ? kWAggWavesPerUser : kWAggWaves;
    const size_t lds = (size_t)kWAccWords * sizeof(double) + (lay.per_user_books ? (size_t)nwaves * kWTabsShort : sizeof(WideTabs));
    const void *fn = lay.per_user_books ? reinterpret_cast<const void *>(&k_aggregate_wide<true>)
                                        : reinterpret_cast<const void *>(&k_aggregate_wide<false>);
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);   // 71 KB or 50 KB
    if (e != hipSuccess) return e;
    ProfScope prof(K_AGGREGATE, s);
    if (lay.per_user_books)
        hipLaunchKernelGGL(k_aggregate_wide<true>, dim3((uint32_t)lay.nchunks), dim3(64 * nwaves), lds, s, lay, a.words,
                           a.words_stride, a.chunk_offset, a.sub_bits, books, a.out, a.model, a.eta, a.status);
    else
        hipLaunchKernelGGL(k_aggregate_wide<false>, dim3((uint32_t)lay.nchunks), dim3(64 * nwaves), lds, s, lay, a.words,
                           a.words_stride, a.chunk_offset, a.sub_bits, books, a.out, a.model, a.eta, a.status);
    return hipGetLastError();
}

}  // namespace co3
