// PS side (Sec. II-B (iv); Algorithm 1 lines 13-14): invert h_Hf for every user's stream and
// form (1/U) sum_u ghat^(u), eq. (aggregate hat) without the learning rate.
//
// One wavefront per chunk; lane j owns sub-chunk j (64 elements), whose start is the chunk's
// bit offset plus the prefix sum of the sub-chunk bit counts.  Codes of up to kDecBits bits are
// resolved by one LDS table lookup; longer ones by the canonical first-code search.  Decoded
// symbols are staged in LDS so that global stores are coalesced across the wave.
#include "co3_internal.h"
#include "quantize_math.h"

namespace co3 {

constexpr int kStageStride = 17;  // words per staged sub-chunk row (16 + 1: spreads LDS banks)

__device__ inline uint32_t find_chunk_segment_d(const SegDev *segs, uint32_t nseg, uint64_t chunk)
{
    uint32_t lo = 0, hi = nseg;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (segs[mid].chunk_start <= chunk) lo = mid; else hi = mid;
    }
    return lo;
}

__device__ inline uint32_t wave_exclusive_scan_u32(uint32_t x)
{
    const int lane = threadIdx.x & 63;
    uint32_t incl = x;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t y = __shfl_up(incl, o, 64);
        if (lane >= o) incl += y;
    }
    return incl - x;
}

__device__ inline uint32_t load_word(const uint32_t *w, uint64_t i, uint64_t limit)
{
    return i < limit ? w[i] : 0u;
}

// Decode `cnt` (<= 64) symbols of one sub-chunk starting at bit `p0` of stream `w`; symbols go
// to stage_row[0..16] (4 per word).  Returns the number of bits consumed, or ~0u if a prefix
// matched no codeword.
__device__ inline uint32_t decode_subchunk(const uint32_t *__restrict__ w, uint64_t limit, uint64_t p0, int cnt,
                                           const uint16_t *s_dec, const BookDev &book, uint32_t *stage_row)
{
    uint64_t wi = p0 >> 5;
    uint32_t sh = (uint32_t)(p0 & 31u);
    uint64_t window = (((uint64_t)load_word(w, wi, limit) << 32) | load_word(w, wi + 1, limit)) << sh;
    uint32_t avail = 64u - sh;
    wi += 2;
    uint32_t consumed = 0, packed = 0;
    for (int j = 0; j < cnt; ++j) {
        if (avail < 32u) {
            window |= (uint64_t)load_word(w, wi++, limit) << (32u - avail);
            avail += 32u;
        }
        const uint32_t e = s_dec[window >> (64 - kDecBits)];
        uint32_t L = e >> 8, s = e & 0xffu;
        if (L == 0u) {
            // long code: exact 64-bit window at the current position, canonical search
            const uint64_t pos = p0 + consumed;
            const uint64_t i0 = pos >> 5;
            const uint32_t s0 = (uint32_t)(pos & 31u);
            uint64_t full = (((uint64_t)load_word(w, i0, limit) << 32) | load_word(w, i0 + 1, limit)) << s0;
            if (s0) full |= (uint64_t)(load_word(w, i0 + 2, limit) >> (32u - s0));
            const uint32_t maxlen = book.maxlen;
            for (uint32_t l = kDecBits + 1; l <= maxlen; ++l) {
                const uint32_t n_l = book.count[l];
                if (!n_l) continue;
                const uint64_t c = full >> (64u - l);
                const uint64_t f = book.first[l];
                if (c >= f && c - f < (uint64_t)n_l) {
                    L = l;
                    s = book.sorted[book.offset[l] + (uint32_t)(c - f)];
                    break;
                }
            }
            if (L == 0u) return ~0u;
            consumed += L;
            const uint64_t np = pos + L;
            wi = np >> 5;
            sh = (uint32_t)(np & 31u);
            window = (((uint64_t)load_word(w, wi, limit) << 32) | load_word(w, wi + 1, limit)) << sh;
            avail = 64u - sh;
            wi += 2;
        } else {
            window <<= L;
            avail -= L;
            consumed += L;
        }
        packed |= s << (8 * (j & 3));
        if ((j & 3) == 3) { stage_row[j >> 2] = packed; packed = 0; }
    }
    if (cnt & 3) stage_row[cnt >> 2] = packed;
    return consumed;
}

struct ChunkGeom {
    uint32_t seg;
    uint32_t n;       // elements in the chunk
    uint64_t e0;      // first element
    int32_t book;     // table id within a user's set
};

__device__ inline ChunkGeom chunk_geom(const Layout &lay, uint64_t c)
{
    ChunkGeom g;
    g.seg = find_chunk_segment_d(lay.segs, lay.nseg, c);
    const SegDev sd = lay.segs[g.seg];
    g.e0 = sd.offset + (c - sd.chunk_start) * kChunk;
    const uint64_t left = sd.offset + sd.length - g.e0;
    g.n = left < (uint64_t)kChunk ? (uint32_t)left : (uint32_t)kChunk;
    g.book = sd.book;
    return g;
}

// Decode the lane's sub-chunk of user u, chunk c into the LDS stage; flags corrupt sub-chunks.
__device__ inline void decode_user_chunk(const Layout &lay, const ChunkGeom &g, uint64_t c, uint32_t u,
                                         const uint32_t *__restrict__ words, uint64_t words_stride,
                                         const uint64_t *__restrict__ chunk_offset,
                                         const uint16_t *__restrict__ sub_bits, const BookDev &book,
                                         const uint16_t *s_dec, uint32_t *s_stage, uint64_t *status)
{
    const uint32_t lane = threadIdx.x & 63;
    const uint64_t off = chunk_offset[(uint64_t)u * (lay.nchunks + 1) + c];
    const uint32_t sb = sub_bits[((uint64_t)u * lay.nchunks + c) * kSubsPerChunk + lane];
    const uint64_t p0 = off + wave_exclusive_scan_u32(sb);
    const int first_elem = (int)lane * kSub;
    const int cnt = (int)g.n - first_elem < 0 ? 0 : ((int)g.n - first_elem > kSub ? kSub : (int)g.n - first_elem);
    const uint32_t *w = words + (uint64_t)u * words_stride;
    const uint32_t used = decode_subchunk(w, words_stride, p0, cnt, s_dec, book, s_stage + lane * kStageStride);
    if (used != sb || (off & 31u) || p0 + sb > words_stride * 32ull)
        atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CORRUPT), 1ull);
}

__global__ __launch_bounds__(64) void k_decode(Layout lay, const uint32_t *__restrict__ words, uint64_t words_stride,
                                               const uint64_t *__restrict__ chunk_offset,
                                               const uint16_t *__restrict__ sub_bits,
                                               const BookDev *__restrict__ books, uint8_t *__restrict__ sym,
                                               uint64_t sym_stride, float *__restrict__ q, uint64_t q_stride,
                                               uint64_t *__restrict__ status)
{
    __shared__ uint16_t s_dec[kDecEntries];
    __shared__ uint32_t s_stage[kSubsPerChunk * kStageStride];
    const uint32_t lane = threadIdx.x;
    const uint64_t c = blockIdx.x;
    const uint32_t u = blockIdx.y;
    const ChunkGeom g = chunk_geom(lay, c);
    const BookDev &book = books[(lay.per_user_books ? u * lay.books_per_user : 0u) + (uint32_t)g.book];
    for (int i = lane; i < kDecEntries / 2; i += 64)
        reinterpret_cast<uint32_t *>(s_dec)[i] = reinterpret_cast<const uint32_t *>(book.dec)[i];
    __syncthreads();
    decode_user_chunk(lay, g, c, u, words, words_stride, chunk_offset, sub_bits, book, s_dec, s_stage, status);
    __syncthreads();
    const uint8_t *stage_b = reinterpret_cast<const uint8_t *>(s_stage);
    if (sym) {
        uint8_t *dst = sym + (uint64_t)u * sym_stride + g.e0;
        if ((reinterpret_cast<uintptr_t>(dst) & 3u) == 0) {
            for (uint32_t e = 4 * lane; e < g.n; e += 256) {
                const uint32_t wv = s_stage[(e >> 6) * kStageStride + ((e & 63u) >> 2)];
                if (e + 3 < g.n) *reinterpret_cast<uint32_t *>(dst + e) = wv;
                else for (uint32_t b = 0; e + b < g.n; ++b) dst[e + b] = (uint8_t)(wv >> (8 * b));
            }
        } else {
            for (uint32_t e = lane; e < g.n; e += 64)
                dst[e] = stage_b[(e >> 6) * (kStageStride * 4) + (e & 63u)];
        }
    }
    if (q) {
        const int bias = lay.bias[(uint64_t)u * lay.nseg + g.seg];
        float *dst = q + (uint64_t)u * q_stride + g.e0;
        for (uint32_t e = lane; e < g.n; e += 64) {
            const uint32_t s = stage_b[(e >> 6) * (kStageStride * 4) + (e & 63u)];
            dst[e] = __uint_as_float(symbol_value_bits(s, lay.E, lay.M, bias));
        }
    }
}

__global__ __launch_bounds__(64) void k_aggregate(Layout lay, const uint32_t *__restrict__ words,
                                                  uint64_t words_stride, const uint64_t *__restrict__ chunk_offset,
                                                  const uint16_t *__restrict__ sub_bits,
                                                  const BookDev *__restrict__ books, float *__restrict__ out,
                                                  uint64_t *__restrict__ status)
{
    __shared__ uint16_t s_dec[kDecEntries];
    __shared__ uint32_t s_stage[kSubsPerChunk * kStageStride];
    const uint32_t lane = threadIdx.x;
    const uint64_t c = blockIdx.x;
    const ChunkGeom g = chunk_geom(lay, c);
    double acc[kSub];
#pragma unroll
    for (int i = 0; i < kSub; ++i) acc[i] = 0.0;
    int loaded_book = -1;
    for (uint32_t u = 0; u < lay.U; ++u) {
        const int bi = (int)((lay.per_user_books ? u * lay.books_per_user : 0u) + (uint32_t)g.book);
        const BookDev &book = books[bi];
        if (bi != loaded_book) {
            __syncthreads();
            for (int i = lane; i < kDecEntries / 2; i += 64)
                reinterpret_cast<uint32_t *>(s_dec)[i] = reinterpret_cast<const uint32_t *>(book.dec)[i];
            loaded_book = bi;
        }
        __syncthreads();
        decode_user_chunk(lay, g, c, u, words, words_stride, chunk_offset, sub_bits, book, s_dec, s_stage, status);
        __syncthreads();
        const int bias = lay.bias[(uint64_t)u * lay.nseg + g.seg];
        // lane owns elements 256*it + 4*lane + b: rows 4*it + lane/16, word lane%16
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            const uint32_t wv = s_stage[(4 * it + (lane >> 4)) * kStageStride + (lane & 15u)];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const uint32_t s = (wv >> (8 * b)) & 0xffu;
                acc[4 * it + b] += (double)__uint_as_float(symbol_value_bits(s, lay.E, lay.M, bias));
            }
        }
    }
    const double inv_u = 1.0 / (double)lay.U;
    float *dst = out + g.e0;
#pragma unroll
    for (int it = 0; it < 16; ++it) {
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const uint32_t e = 256u * it + 4u * lane + b;
            if (e < g.n) dst[e] = (float)(acc[4 * it + b] * inv_u);
        }
    }
}

hipError_t launch_decode(const Layout &lay, const co3_decode_args &a, const BookDev *books, hipStream_t s)
{
    if (lay.U == 0 || lay.nchunks == 0) return hipSuccess;
    const uint64_t sym_stride = (lay.d + 15) & ~(uint64_t)15;
    hipLaunchKernelGGL(k_decode, dim3((uint32_t)lay.nchunks, lay.U), dim3(64), 0, s, lay, a.words, a.words_stride,
                       a.chunk_offset, a.sub_bits, books, a.symbols, sym_stride, a.q, a.q_stride, a.status);
    return hipGetLastError();
}

hipError_t launch_aggregate(const Layout &lay, const co3_aggregate_args &a, const BookDev *books, hipStream_t s)
{
    if (lay.U == 0 || lay.nchunks == 0) return hipSuccess;
    hipLaunchKernelGGL(k_aggregate, dim3((uint32_t)lay.nchunks), dim3(64), 0, s, lay, a.words, a.words_stride,
                       a.chunk_offset, a.sub_bits, books, a.out, a.status);
    return hipGetLastError();
}

}  // namespace co3
