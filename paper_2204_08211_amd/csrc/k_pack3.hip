// h_Hf: element-wise Huffman coding of the quantized symbols into one binary string per user
// (Sec. II-B (iii), Sec. IV-A (ii); Algorithm 1 line 9).  r, the length the paper's
// communication overhead counts, is the sum of the codeword lengths.
//
// Container: codewords in element order, MSB-first in 32-bit words.  A chunk (4096 elements,
// restarting at each layer) starts on a 32-bit boundary, so workgroups own disjoint words of
// the output and no global atomics are needed.  Three steps:
//   k_pack_chunks<false>  code lengths -> bits per sub-chunk and per chunk
//   k_scan_chunks         exclusive scan of the 32-bit-rounded chunk sizes (64-bit offsets)
//   k_pack_chunks<true>   concatenate the codewords in LDS, copy the words out coalesced
#include "co3_internal.h"

namespace co3 {
namespace three_pass {

constexpr int kPkThreads = 256;
constexpr int kPkPerThread = kChunk / kPkThreads;  // 16 symbols per thread
constexpr int kBitWords = kChunk * CO3_MAX_CODE_LEN / 32;

__device__ inline uint32_t find_chunk_segment(const SegDev *segs, uint32_t nseg, uint64_t chunk)
{
    uint32_t lo = 0, hi = nseg;  // segs[nseg].chunk_start = nchunks > chunk
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (segs[mid].chunk_start <= chunk) lo = mid; else hi = mid;
    }
    return lo;
}

__device__ inline uint32_t wave_inclusive_scan(uint32_t x)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t y = __shfl_up(x, o, 64);
        if (lane >= o) x += y;
    }
    return x;
}

template <bool kPack>
__global__ __launch_bounds__(kPkThreads) void k_pack_chunks(
    Layout lay, const uint8_t *__restrict__ sym, uint64_t sym_stride, const BookDev *__restrict__ books,
    uint32_t *__restrict__ chunk_bits, const uint64_t *__restrict__ chunk_offset,
    uint16_t *__restrict__ sub_bits, uint32_t *__restrict__ words, uint64_t words_stride,
    uint64_t *__restrict__ status)
{
    __shared__ uint32_t s_sym[kChunk / 4 + 8];
    __shared__ uint32_t s_fast[kMaxA];
    __shared__ uint32_t s_wave[kPkThreads / 64];
    __shared__ uint32_t s_bits[kPack ? kBitWords + 1 : 1];

    const uint32_t t = threadIdx.x;
    const uint64_t c = blockIdx.x;
    const uint32_t u = blockIdx.y;
    const uint32_t seg = find_chunk_segment(lay.segs, lay.nseg, c);
    const SegDev sd = lay.segs[seg];
    const uint64_t e0 = sd.offset + (c - sd.chunk_start) * kChunk;
    const uint64_t left = sd.offset + sd.length - e0;
    const uint32_t n = left < (uint64_t)kChunk ? (uint32_t)left : (uint32_t)kChunk;
    const BookDev &book = books[(lay.per_user_books ? u * lay.books_per_user : 0u) + (uint32_t)sd.book];

    s_fast[t] = book.fast[t];

    // stage the chunk's symbol bytes as aligned dwords
    const uint64_t byte0 = (uint64_t)u * sym_stride + e0;
    const uint32_t shift = (uint32_t)(byte0 & 3u);
    const uint32_t *src = reinterpret_cast<const uint32_t *>(sym + (byte0 - shift));
    const uint32_t ndw = (shift + n + 3u) >> 2;
    for (uint32_t i = t; i < ndw; i += kPkThreads) s_sym[i] = src[i];
    __syncthreads();

    // this thread's 16 consecutive symbols
    uint32_t dw[5];
#pragma unroll
    for (int k = 0; k < 5; ++k) dw[k] = s_sym[4 * t + k];
    uint32_t sb[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
        sb[k] = (uint32_t)((((uint64_t)dw[k + 1] << 32) | dw[k]) >> (8 * shift));
    const int first_elem = (int)t * kPkPerThread;
    const int cnt = (int)n - first_elem < 0 ? 0 : ((int)n - first_elem > kPkPerThread ? kPkPerThread : (int)n - first_elem);

    uint32_t ent[kPkPerThread];
    uint32_t total = 0, nocode = 0;
#pragma unroll
    for (int j = 0; j < kPkPerThread; ++j) {
        const uint32_t s = (sb[j >> 2] >> (8 * (j & 3))) & 0xffu;
        uint32_t e = (j < cnt) ? s_fast[s] : 0u;
        uint32_t L = e >> 24;
        if (L == kFastSlow) L = book.len[s];
        if (j < cnt && L == 0u) ++nocode;
        total += L;
        ent[j] = (e & 0x00ffffffu) | (L << 24);  // length field now exact (<= 64); low bits valid if L <= 24
    }

    // exclusive scan of the per-thread bit counts over the workgroup
    const uint32_t incl_w = wave_inclusive_scan(total);
    const uint32_t lane = t & 63, wave = t >> 6;
    if (lane == 63) s_wave[wave] = incl_w;
    __syncthreads();
    uint32_t wave_base = 0, chunk_total = 0;
#pragma unroll
    for (uint32_t k = 0; k < kPkThreads / 64; ++k) {
        if (k < wave) wave_base += s_wave[k];
        chunk_total += s_wave[k];
    }
    const uint32_t incl = wave_base + incl_w;
    const uint32_t excl = incl - total;

    if (!kPack) {
        // bits of each sub-chunk (4 threads) and of the chunk
        const uint32_t hi = __shfl(incl, (int)(lane | 3u), 64);
        const uint32_t lo = __shfl(excl, (int)(lane & ~3u), 64);
        if ((t & 3u) == 0u)
            sub_bits[((uint64_t)u * lay.nchunks + c) * kSubsPerChunk + (t >> 2)] = (uint16_t)(hi - lo);
        if (t == 0) chunk_bits[(uint64_t)u * lay.nchunks + c] = chunk_total;
        if (nocode)
            atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_NOCODE), (unsigned long long)nocode);
        return;
    } else {
        const uint32_t nwords = (chunk_total + 31u) >> 5;
        for (uint32_t i = t; i <= nwords; i += kPkThreads) s_bits[i] = 0;
        __syncthreads();

        uint32_t wi = excl >> 5;        // word receiving the next completed 32 bits
        uint32_t np = excl & 31u;       // bits pending in acc (the leading np bits belong to earlier threads)
        uint64_t acc = 0;
        bool first = true;
        auto append = [&](uint64_t code, uint32_t L) {  // L <= 32, np < 32
            acc = (acc << L) | code;
            np += L;
            if (np >= 32u) {
                np -= 32u;
                const uint32_t w = (uint32_t)(acc >> np);
                if (first) { atomicOr(&s_bits[wi], w); first = false; }
                else s_bits[wi] = w;
                ++wi;
            }
        };
#pragma unroll
        for (int j = 0; j < kPkPerThread; ++j) {
            const uint32_t L = ent[j] >> 24;
            if (L <= (uint32_t)kFastLen) {
                if (L) append(ent[j] & 0x00ffffffu, L);
            } else {
                const uint32_t s = (sb[j >> 2] >> (8 * (j & 3))) & 0xffu;
                const uint64_t code = book.code[s];
                if (L > 32u) { append(code >> 32, L - 32u); append(code & 0xffffffffull, 32u); }
                else append(code, L);
            }
        }
        if (np) atomicOr(&s_bits[wi], (uint32_t)(acc << (32u - np)));
        __syncthreads();

        const uint64_t off_words = chunk_offset[(uint64_t)u * (lay.nchunks + 1) + c] >> 5;
        if (off_words + nwords > words_stride) {
            if (t == 0) atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CAPACITY), 1ull);
            return;
        }
        uint32_t *dst = words + (uint64_t)u * words_stride + off_words;
        for (uint32_t i = t; i < nwords; i += kPkThreads) dst[i] = s_bits[i];
    }
}

// Exclusive scan of the chunks' sizes (rounded up to 32 bits) of one user; payload_bits = r.
constexpr int kScanThreads = 1024;
__global__ __launch_bounds__(kScanThreads) void k_scan_chunks(uint64_t nchunks, const uint32_t *__restrict__ chunk_bits,
                                                            uint64_t *__restrict__ chunk_offset,
                                                            uint64_t *__restrict__ payload_bits)
{
    __shared__ uint32_t s_wave[kScanThreads / 64];
    __shared__ uint32_t s_pay[kScanThreads / 64];
    const uint32_t u = blockIdx.x, t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const uint32_t *cb = chunk_bits + (uint64_t)u * nchunks;
    uint64_t *co = chunk_offset + (uint64_t)u * (nchunks + 1);
    uint64_t running = 0, payload = 0;
    for (uint64_t base = 0; base < nchunks; base += kScanThreads) {
        const uint64_t i = base + t;
        const uint32_t b = (i < nchunks) ? cb[i] : 0u;
        const uint32_t a = (b + 31u) & ~31u;
        const uint32_t incl_w = wave_inclusive_scan(a);
        uint32_t pay = b;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) pay += __shfl_xor(pay, o, 64);
        __syncthreads();  // previous iteration's reads of s_wave are done
        if (lane == 63) { s_wave[wave] = incl_w; s_pay[wave] = pay; }
        __syncthreads();
        uint32_t wave_base = 0, tot = 0, ptot = 0;
        for (uint32_t k = 0; k < kScanThreads / 64; ++k) {
            if (k < wave) wave_base += s_wave[k];
            tot += s_wave[k];
            ptot += s_pay[k];
        }
        if (i < nchunks) co[i] = running + wave_base + incl_w - a;
        running += tot;
        payload += ptot;
    }
    if (t == 0) { co[nchunks] = running; payload_bits[u] = payload; }
}

}  // namespace three_pass
using namespace three_pass;

hipError_t launch_pack3(const Layout &lay, const co3_encode_args &a, const BookDev *books, const EncodeWs &ws,
                       hipStream_t s)
{
    if (lay.U == 0) return hipSuccess;
    const uint64_t sym_stride = (lay.d + 15) & ~(uint64_t)15;
    if (lay.nchunks) {
        ProfScope prof(K_CHUNK_BITS, s);
        hipLaunchKernelGGL(k_pack_chunks<false>, dim3((uint32_t)lay.nchunks, lay.U), dim3(kPkThreads), 0, s, lay,
                           a.symbols, sym_stride, books, ws.chunk_bits, a.chunk_offset, a.sub_bits, a.words,
                           a.words_stride, a.status);
    }
    {
    ProfScope prof(K_SCAN, s);
    hipLaunchKernelGGL(k_scan_chunks, dim3(lay.U), dim3(kScanThreads), 0, s, lay.nchunks, ws.chunk_bits,
                       a.chunk_offset, a.payload_bits);
    }
    if (lay.nchunks) {
        ProfScope prof(K_PACK, s);
        hipLaunchKernelGGL(k_pack_chunks<true>, dim3((uint32_t)lay.nchunks, lay.U), dim3(kPkThreads), 0, s, lay,
                           a.symbols, sym_stride, books, ws.chunk_bits, a.chunk_offset, a.sub_bits, a.words,
                           a.words_stride, a.status);
    }
    return hipGetLastError();
}

}  // namespace co3
