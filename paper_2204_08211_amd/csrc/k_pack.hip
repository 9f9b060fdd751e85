// h_Hf: element-wise Huffman coding of the quantized symbols into one binary string per user
// (Sec. II-B (iii), Sec. IV-A (ii); Algorithm 1 line 9).  r, the length the paper's
// communication overhead counts, is the sum of the codeword lengths.
//
// Container: codewords in element order, MSB-first in 32-bit words.  A chunk (4096 elements,
// restarting at each layer) starts on a 32-bit boundary, so wavefronts own disjoint words of the
// output and no global atomics touch the stream.
//
// A wavefront owns a chunk and lane j owns sub-chunk j (64 elements), exactly as in the decoder;
// nothing in these kernels needs a workgroup barrier.  Three steps:
//   k_pack_wave<false>  code lengths -> bits per sub-chunk (the lane's sum) and per chunk
//   k_scan_chunks       exclusive scan of the 32-bit-rounded chunk sizes (64-bit offsets)
//   k_pack_wave<true>   every lane appends its 64 codewords at its bit offset inside an LDS
//                       window (the offset is the wave prefix sum of the sub-chunk bits), then the
//                       wavefront copies the window's words out coalesced
// The symbols of a chunk are staged in LDS in rows of 16 + 1 words so that every lane reads its
// own row without bank conflicts; once they sit in registers the same LDS words become the
// output window.
#include "co3_internal.h"

namespace co3 {

constexpr int kPkWaves = 4;                         // wavefronts (chunks) per workgroup
constexpr int kPkThreads = 64 * kPkWaves;
constexpr int kRowWords = 17;                       // 16 words of symbols + 1 pad
constexpr int kStageWords = kSubsPerChunk * kRowWords;  // 1088 words hold a chunk's symbols
constexpr int kWinWords = 1088;                     // LDS window of the output: 8.5 bit/element per pass
constexpr int kSymLoads = (kChunk / 4 + 1 + 63) / 64;  // dword loads per lane to stage a chunk (17)
constexpr uint32_t kPlainFlag = 1u << 31;              // in chunk_bits: full chunk, every code at most kFastLen bits

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

__device__ inline uint32_t wave_sum(uint32_t x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

__device__ inline void wave_sync_lds()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <bool kPack>
__global__ __launch_bounds__(kPkThreads) void k_pack_wave(
    Layout lay, const uint8_t *__restrict__ sym, uint64_t sym_stride, const BookDev *__restrict__ books,
    uint32_t *__restrict__ chunk_bits, const uint64_t *__restrict__ chunk_offset,
    uint16_t *__restrict__ sub_bits, uint32_t *__restrict__ words, uint64_t words_stride,
    uint64_t *__restrict__ status)
{
    __shared__ uint32_t s_stage_all[kPkWaves][kStageWords + 1];
    __shared__ uint32_t s_win_all[kPkWaves][kPack ? kWinWords + 1 : 1];
    __shared__ uint32_t s_fast_all[kPkWaves][kMaxA];

    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t c = (uint64_t)blockIdx.x * kPkWaves + wave;
    const uint32_t u = blockIdx.y;
    if (c >= lay.nchunks) return;  // whole wavefront; no workgroup barriers below
    uint32_t *s_stage = s_stage_all[wave];
    uint32_t *s_win = s_win_all[wave];
    uint32_t *s_fast = s_fast_all[wave];

    const uint32_t seg = find_chunk_segment(lay.segs, lay.nseg, c);
    const SegDev sd = lay.segs[seg];
    const uint64_t e0 = sd.offset + (c - sd.chunk_start) * kChunk;
    const uint64_t left = sd.offset + sd.length - e0;
    const uint32_t n = left < (uint64_t)kChunk ? (uint32_t)left : (uint32_t)kChunk;
    const BookDev &book = books[(lay.per_user_books ? u * lay.books_per_user : 0u) + (uint32_t)sd.book];

    // what the wavefront needs from memory, requested together: table, symbols, (pack) sub-chunk bits
    uint32_t tab[kMaxA / 64];
#pragma unroll
    for (int k = 0; k < kMaxA / 64; ++k) tab[k] = book.fast[lane + 64 * k];
    const uint64_t byte0 = (uint64_t)u * sym_stride + e0;
    const uint32_t shift = (uint32_t)(byte0 & 3u);
    const uint32_t *src = reinterpret_cast<const uint32_t *>(sym + (byte0 - shift));
    const uint32_t ndw = (shift + n + 3u) >> 2;
    uint32_t tmp[kSymLoads];
#pragma unroll
    for (int k = 0; k < kSymLoads; ++k) {
        const uint32_t i = lane + 64u * k;
        tmp[k] = i < ndw ? src[i] : 0u;
    }
    uint32_t my_bits = 0;
    uint64_t off = 0;
    bool all_plain = false;
    if (kPack) {
        my_bits = sub_bits[((uint64_t)u * lay.nchunks + c) * kSubsPerChunk + lane];
        off = chunk_offset[(uint64_t)u * (lay.nchunks + 1) + c];
        all_plain = (chunk_bits[(uint64_t)u * lay.nchunks + c] & kPlainFlag) != 0u;
    }
#pragma unroll
    for (int k = 0; k < kMaxA / 64; ++k) s_fast[lane + 64 * k] = tab[k];
#pragma unroll
    for (int k = 0; k < kSymLoads; ++k) {
        const uint32_t i = lane + 64u * k;
        if (i < kChunk / 4 + 1) s_stage[i + (i >> 4)] = tmp[k];  // rows of 16 words, 17 apart
    }
    const int first = (int)lane * kSub;
    const int cnt = (int)n - first < 0 ? 0 : ((int)n - first > kSub ? kSub : (int)n - first);
    const uint32_t *row = s_stage + kRowWords * lane;   // words 16*lane .. of the staged bytes; word 16 is row[17]

    if (!kPack) {
        wave_sync_lds();
        uint32_t total = 0;
        // A full chunk whose symbols all have codes of at most kFastLen bits needs no per-symbol
        // checks; bit 31 of chunk_bits tells the pack step so.
        bool plain = false;
        if (n == (uint32_t)kChunk) {
            uint32_t lo = 0xffu, hi = 0u;
            uint32_t cur = row[0];
#pragma unroll 4
            for (int jj = 0; jj < kSub / 4; ++jj) {
                const uint32_t nxt = row[jj + 1 + (jj == kSub / 4 - 1 ? 1 : 0)];
                const uint32_t w4 = (uint32_t)((((uint64_t)nxt << 32) | cur) >> (8 * shift));
                cur = nxt;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint32_t L = s_fast[(w4 >> (8 * b)) & 0xffu] >> 24;
                    total += L;
                    lo = lo < L ? lo : L;
                    hi = hi > L ? hi : L;
                }
            }
            plain = lo > 0u && hi < kFastSlow;
        }
        if (!plain) {
            uint32_t nocode = 0;
            total = 0;
            uint32_t cur = row[0];
#pragma unroll 4
            for (int jj = 0; jj < kSub / 4; ++jj) {
                const uint32_t nxt = row[jj + 1 + (jj == kSub / 4 - 1 ? 1 : 0)];
                const uint32_t w4 = (uint32_t)((((uint64_t)nxt << 32) | cur) >> (8 * shift));
                cur = nxt;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint32_t s = (w4 >> (8 * b)) & 0xffu;
                    const bool in = 4 * jj + b < cnt;
                    uint32_t L = in ? (s_fast[s] >> 24) : 0u;
                    if (__builtin_expect(L == kFastSlow, 0)) L = book.len[s];
                    nocode += (in && L == 0u) ? 1u : 0u;
                    total += L;
                }
            }
            if (nocode)
                atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_NOCODE), (unsigned long long)nocode);
        }
        sub_bits[((uint64_t)u * lay.nchunks + c) * kSubsPerChunk + lane] = (uint16_t)total;
        const uint32_t chunk_total = wave_sum(total);
        const bool all_plain = !__any(!plain);
        if (lane == 0) chunk_bits[(uint64_t)u * lay.nchunks + c] = chunk_total | (all_plain ? kPlainFlag : 0u);
        return;
    } else {
        const uint32_t incl = wave_inclusive_scan(my_bits);
        const uint32_t excl = incl - my_bits;
        const uint32_t chunk_total = __shfl(incl, 63, 64);
        const uint32_t nwords = (chunk_total + 31u) >> 5;
        const uint64_t off_words = off >> 5;
        if (off_words + nwords > words_stride) {
            if (lane == 0) atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CAPACITY), 1ull);
            return;
        }
        uint32_t *dst = words + (uint64_t)u * words_stride + off_words;

        // the chunk's words pass through the LDS window, kWinWords at a time (one pass up to
        // 8.5 bit/element); every lane ORs its words in, so neighbours may share a word
        for (uint32_t wbase = 0; wbase < nwords; wbase += kWinWords) {
            const uint32_t wn = nwords - wbase < (uint32_t)kWinWords ? nwords - wbase : (uint32_t)kWinWords;
            for (uint32_t i = lane; i <= wn; i += 64) s_win[i] = 0;
            wave_sync_lds();
            uint32_t wi = (excl >> 5) - wbase;  // window word receiving the next completed 32 bits
            uint32_t np = excl & 31u;           // bits pending in acc (the leading np bits belong to earlier lanes)
            uint64_t acc = 0;
            auto append = [&](uint64_t code, uint32_t L) {  // L <= 32, np < 32
                acc = (acc << L) | code;
                np += L;
                if (np >= 32u) {
                    np -= 32u;
                    if (wi < wn) atomicOr(&s_win[wi], (uint32_t)(acc >> np));  // unsigned: false below the window
                    ++wi;
                }
            };
            uint32_t cur = row[0];
            if (all_plain) {
                // the table entries of the next four symbols are requested before the current four
                // are appended: the appends' LDS atomics keep later look-ups behind them
                uint32_t en[4];
                auto lookup4 = [&](int jj) {
                    const uint32_t nxt = row[jj + 1 + (jj == kSub / 4 - 1 ? 1 : 0)];
                    const uint32_t w4 = (uint32_t)((((uint64_t)nxt << 32) | cur) >> (8 * shift));
                    cur = nxt;
#pragma unroll
                    for (int b = 0; b < 4; ++b) en[b] = s_fast[(w4 >> (8 * b)) & 0xffu];
                };
                lookup4(0);
#pragma unroll 2
                for (int jj = 0; jj < kSub / 4; ++jj) {
                    uint32_t e[4];
#pragma unroll
                    for (int b = 0; b < 4; ++b) e[b] = en[b];
                    if (jj + 1 < kSub / 4) lookup4(jj + 1);
#pragma unroll
                    for (int b = 0; b < 4; ++b) append(e[b] & 0x00ffffffu, e[b] >> 24);
                }
            } else {
#pragma unroll 2
                for (int jj = 0; jj < kSub / 4; ++jj) {
                    const uint32_t nxt = row[jj + 1 + (jj == kSub / 4 - 1 ? 1 : 0)];
                    const uint32_t w4 = (uint32_t)((((uint64_t)nxt << 32) | cur) >> (8 * shift));
                    cur = nxt;
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const uint32_t s = (w4 >> (8 * b)) & 0xffu;
                        const uint32_t e = (4 * jj + b < cnt) ? s_fast[s] : 0u;
                        uint32_t L = e >> 24;
                        uint64_t code = e & 0x00ffffffu;
                        if (__builtin_expect(L == kFastSlow, 0)) {
                            L = book.len[s];
                            code = book.code[s];
                            if (L > 32u) {
                                append(code >> 32, L - 32u);
                                code &= 0xffffffffull;
                                L = 32u;
                            }
                        }
                        if (L) append(code, L);
                    }
                }
            }
            if (np && wi < wn) atomicOr(&s_win[wi], (uint32_t)(acc << (32u - np)));
            wave_sync_lds();
            for (uint32_t i = lane; i < wn; i += 64) __builtin_nontemporal_store(s_win[i], dst + wbase + i);
            wave_sync_lds();
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
        const uint32_t b = (i < nchunks) ? (cb[i] & ~kPlainFlag) : 0u;
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

hipError_t launch_pack(const Layout &lay, const co3_encode_args &a, const BookDev *books, const EncodeWs &ws,
                       hipStream_t s)
{
    if (lay.U == 0) return hipSuccess;
    const uint64_t sym_stride = (lay.d + 15) & ~(uint64_t)15;
    const uint32_t gx = (uint32_t)((lay.nchunks + kPkWaves - 1) / kPkWaves);
    if (lay.nchunks) {
        ProfScope prof(K_CHUNK_BITS, s);
        hipLaunchKernelGGL(k_pack_wave<false>, dim3(gx, lay.U), dim3(kPkThreads), 0, s, lay, a.symbols, sym_stride,
                           books, ws.chunk_bits, a.chunk_offset, a.sub_bits, a.words, a.words_stride, a.status);
    }
    {
        ProfScope prof(K_SCAN, s);
        hipLaunchKernelGGL(k_scan_chunks, dim3(lay.U), dim3(kScanThreads), 0, s, lay.nchunks, ws.chunk_bits,
                           a.chunk_offset, a.payload_bits);
    }
    if (lay.nchunks) {
        ProfScope prof(K_PACK, s);
        hipLaunchKernelGGL(k_pack_wave<true>, dim3(gx, lay.U), dim3(kPkThreads), 0, s, lay, a.symbols, sym_stride,
                           books, ws.chunk_bits, a.chunk_offset, a.sub_bits, a.words, a.words_stride, a.status);
    }
    return hipGetLastError();
}

}  // namespace co3
