// The whole user side in one sweep for a code that is held fixed (Algorithm 1 lines 8-10 with
// the Huffman code designed beforehand, Sec. IV-A (ii)): error correction, fp conversion, memory
// update and Huffman coding without the symbols ever reaching HBM.
//
// HBM traffic per element: read g (4) + read m (4) + write m' (4) + write b (r/d bits).
//
// A workgroup of four wavefronts takes four consecutive chunks of one user:
//   1. wavefront w quantizes chunk w (16 KB of g and of m, requested a quarter at a time with the
//      next quarter in flight while the current one is computed) and leaves the symbols in LDS,
//      in the rows of 16 + 1 words the pack step reads without bank conflicts; the code's tables go
//      to LDS while the first vectors are under way and the code length of every symbol is summed as
//      it is produced, so the chunk's size is known when the sweep ends.  A chunk that starts
//      at an element off the 16-byte grid (layers begin anywhere) takes the same vectors from the
//      boundary below it; only the ragged last chunk of a layer goes element by element;
//   2. the workgroup's 32-bit-rounded size is published and the sizes of all earlier workgroups of
//      the user are collected by a decoupled look-back: every workgroup first publishes its own
//      size, then reads its predecessors' until it meets one that already knows its running total.
//      Workgroups take their position from a ticket counter, so every predecessor is already
//      running and publishes without waiting for anyone: the wait always ends.  It is bounded all
//      the same; a workgroup whose bound runs out marks its entry as stalled, which its successors
//      inherit instead of waiting, writes no stream words and is counted in the status block.
//      An entry is one 64-bit word (flag and size together) and carries everything a successor
//      needs, so it is written and read with relaxed device-scope atomics: ordering fences would
//      make every workgroup write back and invalidate its L2;
//   3. while the look-back's answers travel, lane j of every wavefront codes sub-chunk j: the
//      wavefront-level coder of pack_core.h concatenates the lane's codewords in a private LDS row
//      (which also yields the sub-chunk sizes) and moves the rows to their bit offsets within the
//      chunk (this needs no stream offset: chunks are word-aligned);
//   4. the chunk's words are copied out coalesced at the offset the look-back gave.
#include <atomic>

#include "co3_internal.h"
#include "pack_core.h"
#include "quantize_math.h"

namespace co3 {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kFuCpb = 4;                            // chunks (= wavefronts) per workgroup ...
constexpr int kFuCpbSmall = 1;                       // ... and for inputs too small to fill the device that way
constexpr uint64_t kFuSmallGrid = 2048;              // workgroups of kFuCpb chunks below which the small form is used
constexpr int kFuRow = kPcSymRow;                    // 16 words of symbols + 1 pad
constexpr int kFuStage = kPcSymWords;                // 1088 words hold a chunk's symbols
constexpr int kFuBatch = 4;                          // 16-byte vectors of g (and of m) a lane requests at a time
constexpr int kFuBatches = kChunk / 4 / 64 / kFuBatch; // batches per chunk
constexpr int kFuScalar = 8;                         // element rounds a lane requests together on the element path
static std::atomic<uint32_t> g_spin_limit{CO3_LOOKBACK_POLLS_DEFAULT};  // polls of one predecessor entry before giving up

// look-back entry: flag in the top two bits, size in bits below
constexpr uint64_t kLbAgg = 1ull << 62;      // size of this workgroup alone
constexpr uint64_t kLbPrefix = 2ull << 62;   // size of this workgroup and all before it
constexpr uint64_t kLbStalled = 3ull << 62;
constexpr uint64_t kLbValue = (1ull << 62) - 1;

static_assert(kChunk % (4 * 64 * kFuBatch) == 0, "whole batches per chunk");
static_assert(kChunk % (64 * kFuScalar) == 0, "whole element rounds per chunk");

__device__ inline uint32_t fu_find_chunk_segment(const SegDev *segs, uint32_t nseg, uint64_t chunk)
{
    uint32_t lo = 0, hi = nseg;  // segs[nseg].chunk_start = nchunks > chunk
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (segs[mid].chunk_start <= chunk) lo = mid; else hi = mid;
    }
    return lo;
}

__device__ inline void fu_wave_sync_lds()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroup barrier that orders LDS accesses only: unlike __syncthreads() it does not wait for the
// wavefront's outstanding global stores (the m' vectors just written), which nobody in the
// workgroup reads.
__device__ inline void fu_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// kSR: the stochastic conversion (dither from Philox words of (element, user, seed)) instead of
// the closest representative.
// kWaves: wavefronts per SIMD the register budget is cut for.  Five (a few values spill) is what the streaming of
// whole 16-byte-aligned chunks wants; layers that start at arbitrary elements take the shifted path, which holds
// more state and runs faster at four without spills, and so does the stochastic conversion (1.05 against 1.29 ms).
// kHist: also count the symbols per code table (hist_rep: kHistGlobalRep partial tables, folded afterwards), for
// callers that hold a code but want this round's histogram, e.g. to design the next round's code from it.
template <bool kSR, int kCpb, int kWaves, bool kHist>
__global__ __launch_bounds__(64 * kCpb, kWaves) void k_encode_fused(
    Layout lay, const float *__restrict__ g, const float *m, float *m_out, uint64_t row_stride, float gamma,
    uint64_t seed, const BookDev *__restrict__ books, uint32_t *__restrict__ tickets, uint64_t *lb_state, uint32_t nblk,
    uint32_t spin_limit, uint64_t *__restrict__ chunk_offset, uint16_t *__restrict__ sub_bits,
    uint64_t *__restrict__ payload_bits, uint32_t *__restrict__ words, uint64_t words_stride,
    uint64_t *__restrict__ status, uint64_t *__restrict__ hist_rep)
{
    __shared__ uint32_t s_stage[kCpb][kPcRegion];     // a wavefront's symbols, then its lanes' rows, then its chunk's words
    __shared__ uint32_t s_fast[kCpb][kMaxA];
    __shared__ uint8_t s_len[kCpb][kMaxA];            // code lengths (0: no code), for the chunk's size
    __shared__ uint32_t s_hist[kHist ? kCpb : 1][kHist ? kMaxA : 1];   // a wavefront's symbol counts of its chunk
    __shared__ uint64_t s_e0[kCpb];
    __shared__ uint32_t s_n[kCpb], s_book[kCpb], s_cbits[kCpb];
    __shared__ int32_t s_bias[kCpb];
    __shared__ float s_gain[kCpb][2];
    __shared__ uint64_t s_prefix;
    __shared__ uint32_t s_ticket, s_stalled;

    const uint32_t t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const uint32_t u = blockIdx.y;

    if (t == 0) s_ticket = atomicAdd(&tickets[u], 1u);
    fu_lds_barrier();
    const uint32_t b = s_ticket;  // position among the user's workgroups, < nblk = gridDim.x
    const uint64_t c0 = (uint64_t)b * kCpb;
    const uint32_t nck = lay.nchunks - c0 < (uint64_t)kCpb ? (uint32_t)(lay.nchunks - c0) : (uint32_t)kCpb;

    if (t < (uint32_t)kCpb) {
        uint64_t e0 = 0;
        uint32_t n = 0, bk = 0;
        int32_t bias = 0;
        float gn = 1.0f, gi = 1.0f;
        if (t < nck) {
            const uint64_t c = c0 + t;
            const uint32_t seg = fu_find_chunk_segment(lay.segs, lay.nseg, c);
            const SegDev sd = lay.segs[seg];
            e0 = sd.offset + (c - sd.chunk_start) * kChunk;
            const uint64_t left = sd.offset + sd.length - e0;
            n = left < (uint64_t)kChunk ? (uint32_t)left : (uint32_t)kChunk;
            bk = (lay.per_user_books ? u * lay.books_per_user : 0u) + (uint32_t)sd.book;
            bias = lay.bias[(uint64_t)u * lay.nseg + seg];
            gn = lay.gain[2 * ((uint64_t)u * lay.nseg + seg)];
            gi = lay.gain[2 * ((uint64_t)u * lay.nseg + seg) + 1];
        }
        s_e0[t] = e0; s_n[t] = n; s_book[t] = bk; s_bias[t] = bias; s_gain[t][0] = gn; s_gain[t][1] = gi;
    }
    fu_lds_barrier();

    // ---- 1. wavefront w quantizes chunk w, symbols to LDS ---------------------------------------
    const bool active = wave < nck;
    const uint32_t sign_shift = lay.E + lay.M;
    uint32_t len_sum = 0;   // code lengths of the elements this lane quantizes
    if (active) {
        const uint64_t e0 = s_e0[wave];
        const uint32_t nk = s_n[wave];
        const int bias = s_bias[wave];
        const QConst qc = make_qconst(lay.E, lay.M, bias);
        const float gain = s_gain[wave][0], inv_gain = s_gain[wave][1];   // real-valued scale: (1, 1) unless the plan carries one
        const float *gu = g + (uint64_t)u * row_stride + e0;
        const float *mu = m + (uint64_t)u * row_stride + e0;
        float *mo = m_out + (uint64_t)u * row_stride + e0;
        uint32_t n_nonfinite = 0, n_clamped = 0;
        // The code's tables are requested first and stored to LDS once the first vectors of g and m are under
        // way: the chunk's size is summed while it is quantized, so that it can be published right after.
        uint32_t tab_fast[kMaxA / 64];
#pragma unroll
        for (int r = 0; r < kMaxA / 64; ++r) tab_fast[r] = books[s_book[wave]].fast[lane + 64 * r];
        const uint32_t tab_len = reinterpret_cast<const uint32_t *>(books[s_book[wave]].len)[lane];
        auto tables_to_lds = [&]() {
#pragma unroll
            for (int r = 0; r < kMaxA / 64; ++r) s_fast[wave][lane + 64 * r] = tab_fast[r];
            reinterpret_cast<uint32_t *>(s_len[wave])[lane] = tab_len;
            if constexpr (kHist) {
#pragma unroll
                for (int r = 0; r < kMaxA / 64; ++r) s_hist[wave][lane + 64 * r] = 0u;
            }
            fu_wave_sync_lds();
        };
        const uint8_t *len_tab = s_len[wave];
        // Four elements of a 16-byte vector: symbols packed into a word, new memory, counters and code
        // lengths for the elements `valid` marks (bit j: element j belongs to this chunk).
        auto quant4 = [&](const f4 &gv, const f4 &mv, uint64_t elem, uint32_t valid, f4 &eo, uint32_t &packed) {
            packed = 0;
            Philox4 rw;
            if constexpr (kSR) rw = element_random_words(elem, u, seed);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float v = __fadd_rn(gv[j], __fmul_rn(gamma, mv[j]));
                const float y = __fmul_rn(v, gain);
                uint32_t s, flags;
                float q;
                if constexpr (kSR) quantize_stochastic(y, qc, lay.E, lay.M, bias, sign_shift, rw.w[j], s, q, flags);
                else quantize(y, qc, sign_shift, s, q, flags);
                q = __fmul_rn(q, inv_gain);
                eo[j] = (flags & 1u) ? 0.0f : __fsub_rn(v, q);
                const uint32_t ok = (valid >> j) & 1u;
                n_nonfinite += flags & ok;
                n_clamped += (flags >> 1) & ok;
                len_sum += ok ? (uint32_t)len_tab[s] : 0u;
                if constexpr (kHist) {
                    if (ok) atomicAdd(&s_hist[wave][s], 1u);
                }
                packed |= s << (8 * j);
            }
        };
        // A whole chunk takes a vector path: kFuBatch 16-byte vectors of g and of m per lane at a time,
        // the next batch requested before the current one is computed.
        const uint32_t shift = (uint32_t)(e0 & 3u);
        if (nk == (uint32_t)kChunk && shift == 0) {
            f4 gn[kFuBatch], mn[kFuBatch];
#pragma unroll
            for (int r = 0; r < kFuBatch; ++r) {
                const uint32_t i = 4u * (lane + 64u * r);
                gn[r] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(gu + i));
                mn[r] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(mu + i));
            }
            tables_to_lds();
#pragma unroll 1
            for (int bt = 0; bt < kFuBatches; ++bt) {
                f4 gc[kFuBatch], mc[kFuBatch];
#pragma unroll
                for (int r = 0; r < kFuBatch; ++r) { gc[r] = gn[r]; mc[r] = mn[r]; }
                if (bt + 1 < kFuBatches) {
#pragma unroll
                    for (int r = 0; r < kFuBatch; ++r) {
                        const uint32_t i = 4u * (lane + 64u * (uint32_t)((bt + 1) * kFuBatch + r));
                        gn[r] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(gu + i));
                        mn[r] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(mu + i));
                    }
                }
#pragma unroll
                for (int r = 0; r < kFuBatch; ++r) {
                    const uint32_t dw = lane + 64u * (uint32_t)(bt * kFuBatch + r);  // word of the chunk's symbols
                    f4 eo;
                    uint32_t packed;
                    quant4(gc[r], mc[r], e0 + 4u * dw, 0xfu, eo, packed);
                    __builtin_nontemporal_store(eo, reinterpret_cast<f4 *>(mo + 4u * dw));
                    s_stage[wave][dw + (dw >> 4)] = packed;
                }
            }
        } else if (nk == (uint32_t)kChunk) {
            // A layer may start at any element.  The same vectors, taken from the 16-byte boundary
            // below the chunk: vector k holds the chunk's elements 4k - shift .. 4k - shift + 3, so
            // its symbols fall into words k - 1 and k of the stage (OR-ed in; the stage is cleared
            // first) and the vectors at both ends are partial.
            const float *ga = gu - shift, *ma = mu - shift;
            float *moa = mo - shift;
            f4 gn[kFuBatch], mn[kFuBatch];
#pragma unroll
            for (int r = 0; r < kFuBatch; ++r) {
                const uint32_t i = 4u * (lane + 64u * r);
                gn[r] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(ga + i));
                mn[r] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(ma + i));
            }
            for (uint32_t i = lane; i < (uint32_t)(kFuStage + 1); i += 64) s_stage[wave][i] = 0;
            tables_to_lds();
#pragma unroll 1
            for (int bt = 0; bt < kFuBatches; ++bt) {
                f4 gc[kFuBatch], mc[kFuBatch];
#pragma unroll
                for (int r = 0; r < kFuBatch; ++r) { gc[r] = gn[r]; mc[r] = mn[r]; }
                if (bt + 1 < kFuBatches) {
#pragma unroll
                    for (int r = 0; r < kFuBatch; ++r) {
                        const uint32_t i = 4u * (lane + 64u * (uint32_t)((bt + 1) * kFuBatch + r));
                        gn[r] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(ga + i));
                        mn[r] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(ma + i));
                    }
                }
#pragma unroll
                for (int r = 0; r < kFuBatch; ++r) {
                    const uint32_t k = lane + 64u * (uint32_t)(bt * kFuBatch + r);  // vector, 0 .. 1023
                    const uint32_t valid = k ? 0xfu : (0xfu << shift) & 0xfu;      // vector 0 starts before the chunk
                    f4 eo;
                    uint32_t packed;
                    quant4(gc[r], mc[r], e0 - shift + 4u * k, valid, eo, packed);
                    if (k) {
                        __builtin_nontemporal_store(eo, reinterpret_cast<f4 *>(moa + 4u * k));
                        atomicOr(&s_stage[wave][(k - 1u) + ((k - 1u) >> 4)], packed << (8u * (4u - shift)));
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if ((valid >> j) & 1u) moa[j] = eo[j];
                    }
                    atomicOr(&s_stage[wave][k + (k >> 4)], packed >> (8u * shift));
                }
            }
            if (lane == 0) {
                // vector 1024: the chunk's last `shift` elements
                f4 gv = {0.0f, 0.0f, 0.0f, 0.0f}, mv = {0.0f, 0.0f, 0.0f, 0.0f}, eo;
                for (uint32_t j = 0; j < shift; ++j) { gv[j] = ga[kChunk + j]; mv[j] = ma[kChunk + j]; }
                uint32_t packed;
                quant4(gv, mv, e0 - shift + kChunk, (1u << shift) - 1u, eo, packed);
                for (uint32_t j = 0; j < shift; ++j) moa[kChunk + j] = eo[j];
                const uint32_t last = kChunk / 4 - 1;
                atomicOr(&s_stage[wave][last + (last >> 4)], (packed & ((1u << (8u * shift)) - 1u)) << (8u * (4u - shift)));
            }
        } else {
            // ragged chunk (the end of a layer): a lane takes one element of every 64, kFuScalar rounds requested together; four neighbouring lanes then gather
            // their symbols into one word of the stage
            tables_to_lds();
            for (uint32_t base = 0; base < nk; base += 64u * kFuScalar) {
                float gs[kFuScalar], ms[kFuScalar];
#pragma unroll
                for (int r = 0; r < kFuScalar; ++r) {
                    const uint32_t j = base + lane + 64u * r;
                    gs[r] = j < nk ? gu[j] : 0.0f;
                    ms[r] = j < nk ? mu[j] : 0.0f;
                }
#pragma unroll
                for (int r = 0; r < kFuScalar; ++r) {
                    const uint32_t j = base + lane + 64u * r;  // < kChunk: base is a multiple of 64 kFuScalar
                    const bool in = j < nk;
                    const float v = __fadd_rn(gs[r], __fmul_rn(gamma, ms[r]));
                    const float y = __fmul_rn(v, gain);
                    uint32_t s, flags;
                    float q;
                    if constexpr (kSR)
                        quantize_stochastic(y, qc, lay.E, lay.M, bias, sign_shift,
                                            element_random_words(e0 + j, u, seed).w[(e0 + j) & 3u], s, q, flags);
                    else quantize(y, qc, sign_shift, s, q, flags);
                    q = __fmul_rn(q, inv_gain);
                    if (in) {
                        mo[j] = (flags & 1u) ? 0.0f : __fsub_rn(v, q);
                        n_nonfinite += flags & 1u;
                        n_clamped += (flags >> 1) & 1u;
                        len_sum += (uint32_t)len_tab[s];
                        if constexpr (kHist) atomicAdd(&s_hist[wave][s], 1u);
                    }
                    s = in ? s : 0u;
                    const uint32_t s4 = s | (__shfl_down(s, 1, 64) << 8) | (__shfl_down(s, 2, 64) << 16) |
                                        (__shfl_down(s, 3, 64) << 24);
                    const uint32_t dw = j >> 2;
                    if ((lane & 3u) == 0 && in) s_stage[wave][dw + (dw >> 4)] = s4;
                }
            }
        }
        if (n_nonfinite)
            atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_NONFINITE),
                      (unsigned long long)n_nonfinite);
        if (n_clamped)
            atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CLAMPED), (unsigned long long)n_clamped);
        if constexpr (kHist) {
            // the chunk's counts go to one of the partial tables of its code table
            fu_wave_sync_lds();
            uint64_t *dst = hist_rep + ((uint64_t)(blockIdx.x % kHistGlobalRep) * lay.nbooks + s_book[wave]) * lay.A;
#pragma unroll
            for (int r = 0; r < kMaxA / 64; ++r) {
                const uint32_t bin = lane + 64u * r;
                const uint32_t cnt = s_hist[wave][bin];
                if (cnt && bin < lay.A) atomicAdd(reinterpret_cast<unsigned long long *>(dst + bin), (unsigned long long)cnt);
            }
        }
    }
    // the chunk's size: every lane summed the code lengths of the elements it quantized
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) len_sum += __shfl_xor(len_sum, o, 64);
    if (lane == 0) s_cbits[wave] = len_sum;  // 0 for a wavefront without a chunk
    fu_lds_barrier();                        // also: every wavefront's symbols are staged

    // ---- 2. publish the workgroup's size; request the predecessors' ------------------------------
    uint32_t before = 0;  // 32-bit-rounded sizes of the workgroup's chunks ahead of this wavefront's
    uint32_t own = 0, pay = 0;
#pragma unroll
    for (int k = 0; k < kCpb; ++k) {
        const uint32_t a = (s_cbits[k] + 31u) & ~31u;
        if ((uint32_t)k < wave) before += a;
        own += a;
        pay += s_cbits[k];
    }
    uint64_t *state = lb_state + (uint64_t)u * nblk;
    if (t == 0)
        __hip_atomic_store(&state[b], (b == 0 ? kLbPrefix : kLbAgg) | own, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    // the nearest 64 predecessor entries, requested now and looked at after the coding below
    uint64_t lb_first = kLbPrefix;  // before the first workgroup: running total 0
    if (wave == 0 && (int64_t)b - 1 - (int64_t)lane >= 0)
        lb_first = __hip_atomic_load(&state[b - 1 - lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

    // ---- 3. wavefront = chunk, lane = sub-chunk: the chunk's words, built in LDS ---------------------
    // A chunk starts on a word boundary, so its words do not depend on where it lands in the stream.
    const uint64_t c = c0 + wave;
    const uint32_t n = active ? s_n[wave] : 0u;
    const int first = (int)lane * kSub;
    const int cnt = (int)n - first < 0 ? 0 : ((int)n - first > kSub ? kSub : (int)n - first);
    uint32_t *region = s_stage[wave];
    const uint32_t *fast = s_fast[wave];
    const BookDev &book = books[s_book[wave]];
    uint32_t symw[kSub / 4];
    uint32_t my_bits = 0;
    bool fast_ok = true;
    if (active) {
        const uint32_t *row = region + kFuRow * lane;
#pragma unroll
        for (int jj = 0; jj < kSub / 4; ++jj) symw[jj] = row[jj];
        fu_wave_sync_lds();  // every lane has its symbols: the region is free
        fast_ok = n == (uint32_t)kChunk ? pc_pack_rows<true>(symw, cnt, fast, region, lane, my_bits)
                                        : pc_pack_rows<false>(symw, cnt, fast, region, lane, my_bits);
        if (!fast_ok) {
            uint32_t nocode = 0;
            my_bits = pc_general_count(symw, cnt, fast, book, region, lane, nocode);
            if (nocode)
                atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_NOCODE), (unsigned long long)nocode);
        }
        sub_bits[((uint64_t)u * lay.nchunks + c) * kSubsPerChunk + lane] = (uint16_t)my_bits;
    }
    const uint32_t incl = pc_wave_inclusive_scan(my_bits, lane);
    const uint32_t excl = incl - my_bits;
    const uint32_t chunk_total = __shfl(incl, 63, 64);   // equals s_cbits[wave]: the same lengths, summed in another order
    const uint32_t nwords = (chunk_total + 31u) >> 5;
    if (active && fast_ok) pc_rows_to_window(region, lane, my_bits, excl, nwords);

    if (wave == 0) {
        uint64_t prefix = 0;
        int64_t pos = (int64_t)b - 1;
        bool stalled = false;
        while (pos >= 0) {
            const int64_t idx = pos - (int64_t)lane;
            uint64_t v = kLbPrefix;  // before the first workgroup: running total 0
            if (idx >= 0) {
                uint32_t spins = 0;
                v = pos == (int64_t)b - 1 ? lb_first
                                          : __hip_atomic_load(&state[idx], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                while ((v >> 62) == 0 && spins < spin_limit) {
                    __builtin_amdgcn_s_sleep(1);
                    v = __hip_atomic_load(&state[idx], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    ++spins;
                }
            }
            // lane 0 holds the nearest predecessor; sum up to and including the first running total
            const uint64_t has_prefix = __ballot((v >> 62) == 2);
            const int stop = has_prefix ? (int)__builtin_ctzll(has_prefix) : 63;
            const bool bad = (int)lane <= stop && ((v >> 62) == 0 || (v >> 62) == 3);
            if (__any(bad)) { stalled = true; break; }
            uint64_t val = ((int)lane <= stop) ? (v & kLbValue) : 0ull;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) val += __shfl_xor(val, o, 64);
            prefix += val;
            if (has_prefix) break;
            pos -= 64;
        }
        if (lane == 0) {
            if (stalled) {
                __hip_atomic_store(&state[b], kLbStalled, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_STALLED), 1ull);
            } else if (b != 0) {
                __hip_atomic_store(&state[b], kLbPrefix | (prefix + own), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
            s_prefix = prefix;
            s_stalled = stalled ? 1u : 0u;
            atomicAdd(reinterpret_cast<unsigned long long *>(payload_bits + u), (unsigned long long)pay);
        }
    }
    fu_lds_barrier();
    if (!active || s_stalled) return;  // whole wavefronts; no workgroup barrier below

    // ---- 4. the chunk's words go to their place in the stream -----------------------------------
    const uint64_t off = s_prefix + before;
    if (lane == 0) {
        uint64_t *co = chunk_offset + (uint64_t)u * (lay.nchunks + 1);
        co[c] = off;
        if (c + 1 == lay.nchunks) co[lay.nchunks] = off + ((chunk_total + 31u) & ~31u);
    }
    const uint64_t off_words = off >> 5;
    if (off_words + nwords > words_stride) {
        if (lane == 0) atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CAPACITY), 1ull);
        return;
    }
    uint32_t *dst = words + (uint64_t)u * words_stride + off_words;
    if (fast_ok) {
        for (uint32_t i = lane; i < nwords; i += 64) __builtin_nontemporal_store(region[i], dst + i);
    } else {
        // the general coder: the symbols are back in LDS, the words pass through a small window
        const uint32_t *win = region + kPcSymWords;
        for (uint32_t wbase = 0; wbase < nwords; wbase += kPcWin) {
            const uint32_t wn = nwords - wbase < (uint32_t)kPcWin ? nwords - wbase : (uint32_t)kPcWin;
            pc_general_window(cnt, fast, book, region, lane, excl, wbase, wn);
            for (uint32_t i = lane; i < wn; i += 64) __builtin_nontemporal_store(win[i], dst + wbase + i);
            fu_wave_sync_lds();
        }
    }
}

// Fill kernel for the look-back state and the payload counters (no memset node, so that callers
// may capture the sequence in a graph).
__global__ void k_zero_fused(uint64_t *p, uint64_t n, uint64_t *q, uint64_t nq)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
    if (i < nq) q[i] = 0;
}

// Chunks per workgroup for this layout: fewer when there would be too few workgroups to fill the device.
static int fused_chunks_per_workgroup(const Layout &lay)
{
    const uint64_t groups = (uint64_t)lay.U * ((lay.nchunks + kFuCpb - 1) / kFuCpb);
    return groups < kFuSmallGrid ? kFuCpbSmall : kFuCpb;
}

size_t fused_workspace_bytes(const Layout &lay)
{
    const uint64_t cpb = (uint64_t)fused_chunks_per_workgroup(lay);
    const uint64_t nblk = (lay.nchunks + cpb - 1) / cpb;
    // tickets (one 64-bit slot per user), the look-back entries, the partial symbol-count tables of the
    // histogram option, plus alignment slack
    return (size_t)(((uint64_t)lay.U + (uint64_t)lay.U * nblk + (uint64_t)kHistGlobalRep * lay.nbooks * lay.A) *
                        sizeof(uint64_t) + 512);
}

template <bool kSR, int kCpb, int kWaves, bool kHist>
static void launch_fused_waves(const Layout &lay, const co3_encode_args &a, const BookDev *books, uint32_t *tickets,
                               uint64_t *lb_state, uint32_t nblk, uint64_t *hist_rep, hipStream_t s)
{
    hipLaunchKernelGGL((k_encode_fused<kSR, kCpb, kWaves, kHist>), dim3(nblk, lay.U), dim3(64 * kCpb), 0, s, lay, a.g, a.m,
                       a.m_out, a.row_stride, a.gamma, a.seed, books, tickets, lb_state, nblk, g_spin_limit.load(),
                       a.chunk_offset, a.sub_bits, a.payload_bits, a.words, a.words_stride, a.status, hist_rep);
}

template <bool kSR, int kCpb>
static void launch_fused_variant(const Layout &lay, const co3_encode_args &a, const BookDev *books, uint32_t *tickets,
                                 uint64_t *lb_state, uint32_t nblk, uint64_t *hist_rep, hipStream_t s)
{
    if (a.hist) launch_fused_waves<kSR, kCpb, 4, true>(lay, a, books, tickets, lb_state, nblk, hist_rep, s);
    else if (lay.vec_aligned && !kSR) launch_fused_waves<kSR, kCpb, 5, false>(lay, a, books, tickets, lb_state, nblk, hist_rep, s);
    else launch_fused_waves<kSR, kCpb, 4, false>(lay, a, books, tickets, lb_state, nblk, hist_rep, s);
}

hipError_t launch_encode_fused(const Layout &lay, const co3_encode_args &a, const BookDev *books, hipStream_t s)
{
    if (lay.U == 0) return hipSuccess;
    const int cpb = fused_chunks_per_workgroup(lay);
    const uint64_t nblk = (lay.nchunks + (uint64_t)cpb - 1) / (uint64_t)cpb;
    uint64_t *base = reinterpret_cast<uint64_t *>((reinterpret_cast<uintptr_t>(a.workspace) + 255u) & ~(uintptr_t)255u);
    uint64_t *ticket_slots = base;               // [U], the low 32 bits of each are the counter
    uint64_t *lb_state = base + lay.U;           // [U][nblk]
    uint64_t *hist_rep = lb_state + (uint64_t)lay.U * nblk;   // [kHistGlobalRep][nbooks][A], with a.hist only
    const uint64_t hist_n = (uint64_t)lay.nbooks * lay.A;
    const uint64_t nz = (uint64_t)lay.U + (uint64_t)lay.U * nblk + (a.hist ? (uint64_t)kHistGlobalRep * hist_n : 0);
    {
        ProfScope prof(K_ZERO, s);
        const uint64_t nmax = nz > lay.U ? nz : lay.U;
        hipLaunchKernelGGL(k_zero_fused, dim3((uint32_t)((nmax + 255) / 256)), dim3(256), 0, s, base, nz,
                           a.payload_bits, (uint64_t)lay.U);
    }
    if (lay.nchunks == 0) {
        // nothing to encode: every user's stream is empty; chunk_offset[u][0] = 0
        {
            ProfScope prof(K_ZERO, s);
            hipLaunchKernelGGL(k_zero_fused, dim3((lay.U + 255) / 256), dim3(256), 0, s, a.chunk_offset,
                               (uint64_t)lay.U, a.chunk_offset, (uint64_t)0);
        }
        if (a.hist) return launch_reduce_hist(hist_rep, a.hist, hist_n, s);   // all-zero counts
        return hipGetLastError();
    }
    {
        ProfScope prof(K_FUSED, s);
        uint32_t *tickets = reinterpret_cast<uint32_t *>(ticket_slots);
        const bool sr = a.rounding == CO3_ROUND_STOCHASTIC;
        if (cpb == kFuCpb) {
            if (sr) launch_fused_variant<true, kFuCpb>(lay, a, books, tickets, lb_state, (uint32_t)nblk, hist_rep, s);
            else launch_fused_variant<false, kFuCpb>(lay, a, books, tickets, lb_state, (uint32_t)nblk, hist_rep, s);
        } else {
            if (sr) launch_fused_variant<true, kFuCpbSmall>(lay, a, books, tickets, lb_state, (uint32_t)nblk, hist_rep, s);
            else launch_fused_variant<false, kFuCpbSmall>(lay, a, books, tickets, lb_state, (uint32_t)nblk, hist_rep, s);
        }
    }
    if (a.hist) return launch_reduce_hist(hist_rep, a.hist, hist_n, s);
    return hipGetLastError();
}

}  // namespace co3

extern "C" void co3_set_lookback_polls(uint32_t polls) { co3::g_spin_limit.store(polls); }
