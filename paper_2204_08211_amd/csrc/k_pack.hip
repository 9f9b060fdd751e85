// h_Hf: element-wise Huffman coding of the quantized symbols into one binary string per user
// (Sec. II-B (iii), Sec. IV-A (ii); Algorithm 1 line 9).  r, the length the paper's
// communication overhead counts, is the sum of the codeword lengths.
//
// Container: codewords in element order, MSB-first in 32-bit words.  A chunk (4096 elements,
// restarting at each layer) starts on a 32-bit boundary, so wavefronts own disjoint words of the
// output and no global atomics touch the stream.
//
// Coder for symbols stored by the quantize sweep.  Three steps:
//   k_chunk_bits   sum of the code lengths of every chunk: a wavefront per chunk, coalesced loads, a
//                  byte table of lengths in LDS (k_chunk_bits_hist: the same sums from the per-chunk symbol
//                  counts the quantize sweep writes for single-layer vectors, without touching the symbols)
//   k_scan_chunks  exclusive scan of the 32-bit-rounded chunk sizes (64-bit offsets), payload r
//   k_pack_chunk   a wavefront per chunk, lane j owns sub-chunk j (64 elements), exactly as in the
//                  decoder: the wavefront-level coder of pack_core.h builds the chunk's words in LDS,
//                  which are then copied out coalesced; the lanes' bit counts are the sub-chunk index
// Nothing in these kernels needs a workgroup barrier.
#include "co3_internal.h"
#include "pack_core.h"

namespace co3 {

constexpr int kPkWaves = 4;                         // wavefronts (chunks) per workgroup
constexpr int kPkThreads = 64 * kPkWaves;
constexpr int kSymLoads = (kChunk / 4 + 1 + 63) / 64;  // dword loads per lane to cover a chunk at any byte offset (17)

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
    return pc_wave_inclusive_scan(x, threadIdx.x & 63);
}

__device__ inline uint32_t wave_sum(uint32_t x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

// Where chunk c of user u lies: first symbol byte (within the symbol buffer), element count, code table.
struct PkChunk {
    uint64_t byte0;
    uint32_t n;
    uint32_t book;
};

__device__ inline PkChunk pk_chunk(const Layout &lay, uint64_t c, uint32_t u, uint64_t sym_stride)
{
    const uint32_t seg = find_chunk_segment(lay.segs, lay.nseg, c);
    const SegDev sd = lay.segs[seg];
    const uint64_t e0 = sd.offset + (c - sd.chunk_start) * kChunk;
    const uint64_t left = sd.offset + sd.length - e0;
    PkChunk k;
    k.byte0 = (uint64_t)u * sym_stride + e0;
    k.n = left < (uint64_t)kChunk ? (uint32_t)left : (uint32_t)kChunk;
    k.book = (lay.per_user_books ? u * lay.books_per_user : 0u) + (uint32_t)sd.book;
    return k;
}

// chunk_bits[u][c] = sum of the code lengths of the chunk's symbols (symbols without a code add nothing;
// they are counted where they are coded).  Lane l takes dwords l, l + 64, ... of the chunk's bytes.
__global__ __launch_bounds__(kPkThreads) void k_chunk_bits(Layout lay, const uint8_t *__restrict__ sym, uint64_t sym_stride,
                                                          const BookDev *__restrict__ books,
                                                          uint32_t *__restrict__ chunk_bits)
{
    __shared__ uint8_t s_len_all[kPkWaves][kMaxA];
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t c = (uint64_t)blockIdx.x * kPkWaves + wave;
    const uint32_t u = blockIdx.y;
    if (c >= lay.nchunks) return;  // whole wavefront; no workgroup barriers below
    const PkChunk k = pk_chunk(lay, c, u, sym_stride);
    uint8_t *s_len = s_len_all[wave];
    const uint32_t len4 = reinterpret_cast<const uint32_t *>(books[k.book].len)[lane];
    const uint32_t shift = (uint32_t)(k.byte0 & 3u);
    const uint32_t *src = reinterpret_cast<const uint32_t *>(sym + (k.byte0 - shift));
    const uint32_t ndw = (shift + k.n + 3u) >> 2;
    uint32_t w[kSymLoads];
#pragma unroll
    for (int r = 0; r < kSymLoads; ++r) {
        const uint32_t i = lane + 64u * r;
        w[r] = i < ndw ? __builtin_nontemporal_load(src + i) : 0u;
    }
    reinterpret_cast<uint32_t *>(s_len)[lane] = len4;
    pc_wave_sync_lds();
    uint32_t total = 0;
    if (shift == 0 && k.n == (uint32_t)kChunk) {
#pragma unroll
        for (int r = 0; r < kChunk / 4 / 64; ++r)
#pragma unroll
            for (int b = 0; b < 4; ++b) total += s_len[(w[r] >> (8 * b)) & 0xffu];
    } else {
#pragma unroll
        for (int r = 0; r < kSymLoads; ++r) {
            const uint32_t i = lane + 64u * r;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const uint32_t pos = 4u * i + b;                       // byte within the loaded dwords
                const bool in = pos >= shift && pos < shift + k.n;
                total += in ? s_len[(w[r] >> (8 * b)) & 0xffu] : 0u;
            }
        }
    }
    total = wave_sum(total);
    if (lane == 0) chunk_bits[(uint64_t)u * lay.nchunks + c] = total;
}

// The same sizes from the symbol counts of every chunk that the quantize sweep left behind (single-layer
// vectors): chunk_bits[u][c] = sum over symbols of count x code length.  A wavefront per chunk, four bins per lane.
__global__ __launch_bounds__(kPkThreads) void k_chunk_bits_hist(Layout lay, const uint16_t *__restrict__ chunk_hist,
                                                               const BookDev *__restrict__ books,
                                                               uint32_t *__restrict__ chunk_bits)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t c = (uint64_t)blockIdx.x * kPkWaves + wave;
    const uint32_t u = blockIdx.y;
    if (c >= lay.nchunks) return;
    const BookDev &book = books[(lay.per_user_books ? u * lay.books_per_user : 0u) + (uint32_t)lay.segs[0].book];
    const uint16_t *h = chunk_hist + ((uint64_t)u * lay.nchunks + c) * lay.A;
    uint32_t total = 0;
    for (uint32_t b0 = 4u * lane; b0 < lay.A; b0 += 256u) {   // A is a power of two, at least 8
        const uint2 cnt = *reinterpret_cast<const uint2 *>(h + b0);
        const uint32_t len4 = *reinterpret_cast<const uint32_t *>(book.len + b0);
        total += (cnt.x & 0xffffu) * (len4 & 0xffu) + (cnt.x >> 16) * ((len4 >> 8) & 0xffu) +
                 (cnt.y & 0xffffu) * ((len4 >> 16) & 0xffu) + (cnt.y >> 16) * (len4 >> 24);
    }
    total = wave_sum(total);
    if (lane == 0) chunk_bits[(uint64_t)u * lay.nchunks + c] = total;
}

// The coder proper.  chunk_offset comes from k_scan_chunks.
__global__ __launch_bounds__(kPkThreads) void k_pack_chunk(
    Layout lay, const uint8_t *__restrict__ sym, uint64_t sym_stride, const BookDev *__restrict__ books,
    const uint64_t *__restrict__ chunk_offset, uint16_t *__restrict__ sub_bits, uint32_t *__restrict__ words,
    uint64_t words_stride, uint64_t *__restrict__ status)
{
    __shared__ uint32_t s_region_all[kPkWaves][kPcRegion];
    __shared__ uint32_t s_fast_all[kPkWaves][kMaxA];

    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t c = (uint64_t)blockIdx.x * kPkWaves + wave;
    const uint32_t u = blockIdx.y;
    if (c >= lay.nchunks) return;  // whole wavefront; no workgroup barriers below
    uint32_t *region = s_region_all[wave];
    uint32_t *s_fast = s_fast_all[wave];
    const PkChunk k = pk_chunk(lay, c, u, sym_stride);
    const BookDev &book = books[k.book];

    // what the wavefront needs from memory, requested together: table, symbols, stream offset
    uint32_t tab[kMaxA / 64];
#pragma unroll
    for (int r = 0; r < kMaxA / 64; ++r) tab[r] = book.fast[lane + 64 * r];
    const uint64_t off = chunk_offset[(uint64_t)u * (lay.nchunks + 1) + c];
    uint32_t symw[kSub / 4];   // the lane's 64 symbols, four per word
    {
        // any byte offset, any length: coalesced dwords from the 4-byte boundary below the chunk, staged in LDS
        // rows of 16 + 1 words, from which every lane funnels its 64 bytes
        const uint32_t shift = (uint32_t)(k.byte0 & 3u);
        const uint32_t *src = reinterpret_cast<const uint32_t *>(sym + (k.byte0 - shift));
        const uint32_t ndw = (shift + k.n + 3u) >> 2;
        uint32_t tmp[kSymLoads];
#pragma unroll
        for (int r = 0; r < kSymLoads; ++r) {
            const uint32_t i = lane + 64u * r;
            tmp[r] = i < ndw ? __builtin_nontemporal_load(src + i) : 0u;
        }
#pragma unroll
        for (int r = 0; r < kMaxA / 64; ++r) s_fast[lane + 64 * r] = tab[r];
#pragma unroll
        for (int r = 0; r < kSymLoads; ++r) {
            const uint32_t i = lane + 64u * r;
            if (i < kChunk / 4 + 1) region[i + (i >> 4)] = tmp[r];  // word 1024 lands at 1088
        }
        pc_wave_sync_lds();
        const uint32_t *row = region + kPcSymRow * lane;   // dwords 16 lane .. 16 lane + 15; dword 16 lane + 16 is row[17]
        uint32_t cur = row[0];
#pragma unroll
        for (int jj = 0; jj < kSub / 4; ++jj) {
            const uint32_t nxt = row[jj + 1 + (jj == kSub / 4 - 1 ? 1 : 0)];
            symw[jj] = __builtin_amdgcn_alignbit(nxt, cur, 8u * shift);
            cur = nxt;
        }
        pc_wave_sync_lds();                                // the region is free again
    }
    const int first = (int)lane * kSub;
    const int cnt = (int)k.n - first < 0 ? 0 : ((int)k.n - first > kSub ? kSub : (int)k.n - first);

    uint32_t bits = 0;
    const bool fast_ok = k.n == (uint32_t)kChunk ? pc_pack_rows<true>(symw, cnt, s_fast, region, lane, bits)
                                                 : pc_pack_rows<false>(symw, cnt, s_fast, region, lane, bits);
    if (!fast_ok) {
        uint32_t nocode = 0;
        bits = pc_general_count(symw, cnt, s_fast, book, region, lane, nocode);
        if (nocode)
            atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_NOCODE), (unsigned long long)nocode);
    }
    sub_bits[((uint64_t)u * lay.nchunks + c) * kSubsPerChunk + lane] = (uint16_t)bits;
    const uint32_t incl = wave_inclusive_scan(bits);
    const uint32_t excl = incl - bits;
    const uint32_t chunk_total = __shfl(incl, 63, 64);
    const uint32_t nwords = (chunk_total + 31u) >> 5;
    const uint64_t off_words = off >> 5;
    if (off_words + nwords > words_stride) {
        if (lane == 0) atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CAPACITY), 1ull);
        return;
    }
    uint32_t *dst = words + (uint64_t)u * words_stride + off_words;
    if (fast_ok) {
        pc_rows_to_window(region, lane, bits, excl, nwords);
        for (uint32_t i = lane; i < nwords; i += 64) __builtin_nontemporal_store(region[i], dst + i);
    } else {
        const uint32_t *win = region + kPcSymWords;
        for (uint32_t wbase = 0; wbase < nwords; wbase += kPcWin) {
            const uint32_t wn = nwords - wbase < (uint32_t)kPcWin ? nwords - wbase : (uint32_t)kPcWin;
            pc_general_window(cnt, s_fast, book, region, lane, excl, wbase, wn);
            for (uint32_t i = lane; i < wn; i += 64) __builtin_nontemporal_store(win[i], dst + wbase + i);
            pc_wave_sync_lds();
        }
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
        const uint32_t pay = wave_sum(b);
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

hipError_t launch_scan_chunks(const Layout &lay, const uint32_t *chunk_bits, uint64_t *chunk_offset,
                              uint64_t *payload_bits, hipStream_t s)
{
    if (lay.U == 0) return hipSuccess;
    ProfScope prof(K_SCAN, s);
    hipLaunchKernelGGL(k_scan_chunks, dim3(lay.U), dim3(kScanThreads), 0, s, lay.nchunks, chunk_bits, chunk_offset,
                       payload_bits);
    return hipGetLastError();
}

hipError_t launch_pack(const Layout &lay, const co3_encode_args &a, const BookDev *books, const EncodeWs &ws,
                       hipStream_t s)
{
    if (lay.U == 0) return hipSuccess;
    const uint64_t sym_stride = symbol_row_stride(lay.d);
    const uint32_t gx = (uint32_t)((lay.nchunks + kPkWaves - 1) / kPkWaves);
    if (lay.nchunks) {
        ProfScope prof(K_CHUNK_BITS, s);
        if (ws.chunk_hist)
            hipLaunchKernelGGL(k_chunk_bits_hist, dim3(gx, lay.U), dim3(kPkThreads), 0, s, lay, ws.chunk_hist, books,
                               ws.chunk_bits);
        else
            hipLaunchKernelGGL(k_chunk_bits, dim3(gx, lay.U), dim3(kPkThreads), 0, s, lay, a.symbols, sym_stride, books,
                               ws.chunk_bits);
    }
    if (launch_scan_chunks(lay, ws.chunk_bits, a.chunk_offset, a.payload_bits, s) != hipSuccess) return hipGetLastError();
    if (lay.nchunks) {
        ProfScope prof(K_PACK, s);
        hipLaunchKernelGGL(k_pack_chunk, dim3(gx, lay.U), dim3(kPkThreads), 0, s, lay, a.symbols, sym_stride, books,
                           a.chunk_offset, a.sub_bits, a.words, a.words_stride, a.status);
    }
    return hipGetLastError();
}

}  // namespace co3
