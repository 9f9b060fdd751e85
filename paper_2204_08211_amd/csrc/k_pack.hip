// h_Hf: element-wise Huffman coding of the quantized symbols into one binary string per user
// (Sec. II-B (iii), Sec. IV-A (ii); Algorithm 1 line 9).  r, the length the paper's
// communication overhead counts, is the sum of the codeword lengths.
//
// Container: codewords in element order, MSB-first in 32-bit words.  A chunk (4096 elements,
// restarting at each layer) starts on a 32-bit boundary, so workgroups own disjoint words of
// the output and no global atomics touch the stream.
//
// One kernel, one read of the symbols.  A workgroup takes a ticket (its position in the user's
// sequence), stages the symbols of kCpb consecutive chunks in LDS, sums their code lengths,
// publishes the 32-bit-rounded size of its chunks, obtains the bit offset of its first chunk by
// looking back over the sizes published by its predecessors (decoupled look-back: a predecessor
// either shows its own size or the running total up to and including itself), and then
// concatenates the codewords of each chunk in an LDS window and copies the words out coalesced.
// Tickets make the wait safe: every ticket below a workgroup's own is held by a workgroup that is
// already running and never waits on a later one.  The wait is bounded; on expiry the workgroup
// counts an error in status[CO3_STAT_INTERNAL] and goes on.
#include "co3_internal.h"

namespace co3 {

constexpr int kPkThreads = 256;
constexpr int kPkPerThread = kChunk / kPkThreads;  // 16 symbols per thread and chunk
constexpr int kCpb = 4;                            // chunks per workgroup
constexpr int kWinWords = 2048;                    // LDS window of the output (16 bit/element in one pass)

constexpr uint64_t kLbAgg = 1ull << 62;      // value = size of the workgroup's own chunks
constexpr uint64_t kLbPrefix = 2ull << 62;   // value = total size up to and including the workgroup
constexpr uint64_t kLbValue = (1ull << 62) - 1;

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

// 16 consecutive symbol bytes starting at byte `b` of the staged symbols, as four dwords
__device__ inline void load_symbols16(const uint32_t *s_sym, uint32_t b, uint32_t sb[4])
{
    const uint32_t w = b >> 2, sh = 8u * (b & 3u);
    uint32_t dw[5];
#pragma unroll
    for (int k = 0; k < 5; ++k) dw[k] = s_sym[w + k];
#pragma unroll
    for (int k = 0; k < 4; ++k) sb[k] = (uint32_t)((((uint64_t)dw[k + 1] << 32) | dw[k]) >> sh);
}

__global__ __launch_bounds__(kPkThreads) void k_pack(
    Layout lay, const uint8_t *__restrict__ sym, uint64_t sym_stride, const BookDev *__restrict__ books,
    uint32_t *__restrict__ tickets, uint64_t *__restrict__ lb_state, uint32_t nblk,
    uint64_t *__restrict__ chunk_offset, uint16_t *__restrict__ sub_bits, uint64_t *__restrict__ payload_bits,
    uint32_t *__restrict__ words, uint64_t words_stride, uint64_t *__restrict__ status, uint32_t spin_limit)
{
    __shared__ uint32_t s_sym[kCpb * kChunk / 4 + 8];
    __shared__ uint32_t s_fast[kCpb][kMaxA];
    __shared__ uint32_t s_bits[kWinWords + 1];
    __shared__ uint32_t s_part[kCpb][kPkThreads / 64];
    __shared__ uint32_t s_wave[kPkThreads / 64];
    __shared__ uint32_t s_cn[kCpb], s_coff[kCpb], s_cbook[kCpb], s_cbits[kCpb];
    __shared__ uint64_t s_efirst;
    __shared__ uint64_t s_prefix;
    __shared__ uint32_t s_ticket;

    const uint32_t t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const uint32_t u = blockIdx.y;
    if (t == 0) s_ticket = atomicAdd(&tickets[u], 1u);
    __syncthreads();
    const uint32_t b = s_ticket;                       // position of this workgroup in the user's sequence
    const uint64_t c0 = (uint64_t)b * kCpb;
    const uint32_t nck = (lay.nchunks - c0 < (uint64_t)kCpb) ? (uint32_t)(lay.nchunks - c0) : (uint32_t)kCpb;

    // geometry of the chunks; their elements are contiguous in the user's vector
    if (t < (uint32_t)kCpb) {
        uint32_t n = 0, bk = 0;
        uint64_t e0 = 0;
        if (t < nck) {
            const uint64_t c = c0 + t;
            const uint32_t seg = find_chunk_segment(lay.segs, lay.nseg, c);
            const SegDev sd = lay.segs[seg];
            e0 = sd.offset + (c - sd.chunk_start) * kChunk;
            const uint64_t left = sd.offset + sd.length - e0;
            n = left < (uint64_t)kChunk ? (uint32_t)left : (uint32_t)kChunk;
            bk = (lay.per_user_books ? u * lay.books_per_user : 0u) + (uint32_t)sd.book;
        }
        s_cn[t] = n;
        s_cbook[t] = bk;
        if (t == 0) s_efirst = e0;
    }
    __syncthreads();
    uint32_t n_elems = 0;
#pragma unroll
    for (int k = 0; k < kCpb; ++k) {
        if (t == 0) s_coff[k] = n_elems;
        n_elems += s_cn[k];
        if ((uint32_t)k < nck) s_fast[k][t] = books[s_cbook[k]].fast[t];
    }
    const uint64_t e_first = s_efirst;

    // stage the symbol bytes as aligned dwords: all loads first, then all LDS stores
    const uint64_t byte0 = (uint64_t)u * sym_stride + e_first;
    const uint32_t shift = (uint32_t)(byte0 & 3u);
    const uint32_t *src = reinterpret_cast<const uint32_t *>(sym + (byte0 - shift));
    const uint32_t ndw = (shift + n_elems + 3u) >> 2;
    {
        constexpr int kLoads = (kCpb * kChunk / 4 + kPkThreads) / kPkThreads;  // 17
        uint32_t tmp[kLoads];
#pragma unroll
        for (int k = 0; k < kLoads; ++k) {
            const uint32_t i = t + (uint32_t)k * kPkThreads;
            tmp[k] = i < ndw ? __builtin_nontemporal_load(src + i) : 0u;
        }
#pragma unroll
        for (int k = 0; k < kLoads; ++k) {
            const uint32_t i = t + (uint32_t)k * kPkThreads;
            if (i < ndw) s_sym[i] = tmp[k];
        }
    }
    __syncthreads();

    // pass A: bits of every chunk
    uint32_t nocode = 0;
#pragma unroll
    for (int k = 0; k < kCpb; ++k) {
        uint32_t total = 0;
        if ((uint32_t)k < nck) {
            const int first = (int)t * kPkPerThread;
            const int cn_k = (int)s_cn[k];
            const int cnt = cn_k - first < 0 ? 0 : (cn_k - first > kPkPerThread ? kPkPerThread : cn_k - first);
            if (cnt > 0) {
                uint32_t sb[4];
                load_symbols16(s_sym, shift + s_coff[k] + (uint32_t)first, sb);
#pragma unroll
                for (int j = 0; j < kPkPerThread; ++j) {
                    const uint32_t s = (sb[j >> 2] >> (8 * (j & 3))) & 0xffu;
                    uint32_t L = (j < cnt) ? (s_fast[k][s] >> 24) : 0u;
                    if (L == kFastSlow) L = books[s_cbook[k]].len[s];
                    if (j < cnt && L == 0u) ++nocode;
                    total += L;
                }
            }
        }
        total = wave_sum(total);
        if (lane == 0) s_part[k][wave] = total;
    }
    __syncthreads();
    uint64_t own = 0, pay = 0;   // 32-bit-rounded size of this workgroup's chunks; their payload bits
#pragma unroll
    for (int k = 0; k < kCpb; ++k) {
        uint32_t cb = 0;
#pragma unroll
        for (int w = 0; w < kPkThreads / 64; ++w) cb += s_part[k][w];
        if (t == 0) s_cbits[k] = cb;
        own += (cb + 31u) & ~31u;
        pay += cb;
    }

    // publish, look back, publish the running total
    uint64_t *state = lb_state + (uint64_t)u * nblk;
    if (wave == 0) {
        if (lane == 0)
            __hip_atomic_store(&state[b], (b == 0 ? kLbPrefix : kLbAgg) | own, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        uint64_t prefix = 0;
        int64_t pos = (int64_t)b - 1;
        bool timed_out = false;
        while (pos >= 0) {
            const int64_t idx = pos - (int64_t)lane;
            uint64_t v = kLbPrefix;  // before the first workgroup: total 0
            uint32_t spins = 0;
            if (idx >= 0) {
                v = __hip_atomic_load(&state[idx], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
                while ((v >> 62) == 0 && spins < spin_limit) {
                    __builtin_amdgcn_s_sleep(1);
                    v = __hip_atomic_load(&state[idx], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
                    ++spins;
                }
            }
            if (__any((v >> 62) == 0)) { timed_out = true; break; }
            // nearest predecessor is lane 0; sum up to and including the first running total
            const uint64_t has_prefix = __ballot((v >> 62) == 2);
            const int stop = has_prefix ? (int)__builtin_ctzll(has_prefix) : 63;
            uint64_t val = ((int)lane <= stop) ? (v & kLbValue) : 0ull;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) val += __shfl_xor(val, o, 64);
            prefix += val;
            if (has_prefix) break;
            pos -= 64;
        }
        if (lane == 0) {
            if (timed_out)
                atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_INTERNAL), 1ull);
            if (b != 0)
                __hip_atomic_store(&state[b], kLbPrefix | (prefix + own), __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
            s_prefix = prefix;
            atomicAdd(reinterpret_cast<unsigned long long *>(payload_bits + u), (unsigned long long)pay);
        }
    }
    if (nocode)
        atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_NOCODE), (unsigned long long)nocode);
    __syncthreads();
    uint64_t off = s_prefix;  // bit offset of the first chunk

    // pass B: concatenate the codewords chunk by chunk
#pragma unroll 1
    for (uint32_t k = 0; k < nck; ++k) {
        const uint64_t c = c0 + k;
        const int first = (int)t * kPkPerThread;
        const int cn_k = (int)s_cn[k];
        const int cnt = cn_k - first < 0 ? 0 : (cn_k - first > kPkPerThread ? kPkPerThread : cn_k - first);
        const BookDev &book = books[s_cbook[k]];
        uint32_t sb[4] = {0, 0, 0, 0};
        if (cnt > 0) load_symbols16(s_sym, shift + s_coff[k] + (uint32_t)first, sb);
        uint32_t ent[kPkPerThread];
        uint32_t total = 0;
#pragma unroll
        for (int j = 0; j < kPkPerThread; ++j) {
            const uint32_t s = (sb[j >> 2] >> (8 * (j & 3))) & 0xffu;
            const uint32_t e = (j < cnt) ? s_fast[k][s] : 0u;
            uint32_t L = e >> 24;
            if (L == kFastSlow) L = book.len[s];
            total += L;
            ent[j] = (e & 0x00ffffffu) | (L << 24);  // exact length (<= 64); code bits valid if L <= 24
        }
        const uint32_t incl_w = wave_inclusive_scan(total);
        if (lane == 63) s_wave[wave] = incl_w;
        __syncthreads();
        uint32_t wave_base = 0;
#pragma unroll
        for (uint32_t w = 0; w < kPkThreads / 64; ++w)
            if (w < wave) wave_base += s_wave[w];
        const uint32_t incl = wave_base + incl_w;
        const uint32_t excl = incl - total;
        const uint32_t chunk_total = s_cbits[k];

        // bits of each sub-chunk (4 threads), chunk offset
        const uint32_t hi = __shfl(incl, (int)(lane | 3u), 64);
        const uint32_t lo = __shfl(excl, (int)(lane & ~3u), 64);
        if ((t & 3u) == 0u)
            sub_bits[((uint64_t)u * lay.nchunks + c) * kSubsPerChunk + (t >> 2)] = (uint16_t)(hi - lo);
        if (t == 0) {
            chunk_offset[(uint64_t)u * (lay.nchunks + 1) + c] = off;
            if (c + 1 == lay.nchunks)
                chunk_offset[(uint64_t)u * (lay.nchunks + 1) + c + 1] = off + ((chunk_total + 31u) & ~31u);
        }

        const uint32_t nwords = (chunk_total + 31u) >> 5;
        const uint64_t off_words = off >> 5;
        const bool fits = off_words + nwords <= words_stride;
        if (!fits && t == 0) atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CAPACITY), 1ull);
        uint32_t *dst = words + (uint64_t)u * words_stride + off_words;

        // the chunk's words pass through the LDS window, kWinWords at a time
        for (uint32_t wbase = 0; wbase < nwords && fits; wbase += kWinWords) {
            const uint32_t wn = nwords - wbase < (uint32_t)kWinWords ? nwords - wbase : (uint32_t)kWinWords;
            for (uint32_t i = t; i <= wn; i += kPkThreads) s_bits[i] = 0;
            __syncthreads();
            uint32_t wi = excl >> 5;        // word receiving the next completed 32 bits
            uint32_t np = excl & 31u;       // bits pending in acc (the leading np bits belong to earlier threads)
            uint64_t acc = 0;
            bool firstw = true;
            auto emit = [&](uint32_t w, bool whole) {
                const uint32_t rel = wi - wbase;
                if (rel < wn) {  // unsigned: also false below the window
                    if (firstw || !whole) atomicOr(&s_bits[rel], w);
                    else s_bits[rel] = w;
                }
                firstw = false;
            };
            auto append = [&](uint64_t code, uint32_t L) {  // L <= 32, np < 32
                acc = (acc << L) | code;
                np += L;
                if (np >= 32u) {
                    np -= 32u;
                    emit((uint32_t)(acc >> np), true);
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
            if (np) emit((uint32_t)(acc << (32u - np)), false);
            __syncthreads();
            for (uint32_t i = t; i < wn; i += kPkThreads) __builtin_nontemporal_store(s_bits[i], dst + wbase + i);
            __syncthreads();
        }
        off += (chunk_total + 31u) & ~31u;
    }
}

hipError_t launch_pack(const Layout &lay, const co3_encode_args &a, const BookDev *books, const EncodeWs &ws,
                       hipStream_t s)
{
    if (lay.U == 0) return hipSuccess;
    const uint64_t sym_stride = (lay.d + 15) & ~(uint64_t)15;
    const uint32_t nblk = (uint32_t)((lay.nchunks + kCpb - 1) / kCpb);
    // tickets [U] (as uint64 slots) + look-back state [U][nblk] + payload_bits [U]
    if (launch_zero_u64(ws.lookback, (uint64_t)lay.U * (nblk + 1), s) != hipSuccess) return hipGetLastError();
    if (launch_zero_u64(a.payload_bits, lay.U, s) != hipSuccess) return hipGetLastError();
    if (lay.nchunks == 0) return launch_zero_u64(a.chunk_offset, lay.U, s);
    uint32_t *tickets = reinterpret_cast<uint32_t *>(ws.lookback);
    uint64_t *state = ws.lookback + lay.U;
    ProfScope prof(K_PACK, s);
    hipLaunchKernelGGL(k_pack, dim3(nblk, lay.U), dim3(kPkThreads), 0, s, lay, a.symbols, sym_stride, books, tickets,
                       state, nblk, a.chunk_offset, a.sub_bits, a.payload_bits, a.words, a.words_stride, a.status,
                       ws.spin_limit);
    return hipGetLastError();
}

}  // namespace co3
