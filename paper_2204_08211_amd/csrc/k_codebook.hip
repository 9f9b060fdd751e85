// Huffman code tables built on the device from symbol counts (Sec. IV-A (ii)), one workgroup
// per table, so that an encoder using this round's histogram needs no host round trip.
//
// Same tie rule and canonical form as the host builder: leaves sorted by (weight, symbol),
// internal nodes in creation order, merge the two smallest with leaves first on equal weight.
#include "co3_internal.h"

namespace co3 {

constexpr int kCbThreads = 256;

__global__ __launch_bounds__(kCbThreads) void k_build_books(BookDev *__restrict__ books, uint32_t A,
                                                           const uint64_t *__restrict__ weights,
                                                           uint64_t *__restrict__ status)
{
    BookDev &B = books[blockIdx.x];
    const uint64_t *w = weights + (uint64_t)blockIdx.x * A;
    const int t = threadIdx.x;

    __shared__ uint64_t lw[kMaxA];        // weight of symbol t
    __shared__ uint64_t nw[2 * kMaxA];    // node weights: sorted leaves, then internal nodes
    __shared__ int parent[2 * kMaxA];
    __shared__ uint32_t leaf_sym[kMaxA];  // sorted leaf -> symbol
    __shared__ uint32_t slen[kMaxA];      // symbol -> length
    __shared__ uint32_t cnt[65], off[65];
    __shared__ uint64_t first[65];
    __shared__ uint32_t sorted[kMaxA];
    __shared__ int err;

    const uint64_t myw = (t < (int)A) ? w[t] : 0;
    lw[t] = myw;
    slen[t] = 0;
    parent[t] = -1;
    parent[t + kMaxA] = -1;
    if (t < 65) { cnt[t] = 0; off[t] = 0; first[t] = 0; }
    if (t == 0) err = 0;
    __syncthreads();
    // 2^64 - 1 marks an exhausted queue in the merge below; as a weight it is refused, like the
    // host builder refuses it (the table's weights would sum to 2^64 - 1 or more)
    if (myw == ~0ull) err = 1;
    const int n = __syncthreads_count(myw > 0);

    // rank of this leaf in (weight, symbol) order among the active symbols
    if (myw > 0) {
        int rank = 0;
#pragma unroll 8
        for (int j = 0; j < (int)A; ++j) {
            const uint64_t wj = lw[j];
            rank += (int)((wj != 0) & ((wj < myw) | ((wj == myw) & (j < t))));
        }
        nw[rank] = myw;
        leaf_sym[rank] = t;
    }
    __syncthreads();

    if (t == 0 && n >= 2 && !err) {
        // the two front entries of each queue live in registers, so that the load refilling a queue
        // is not needed before the pick after next; an exhausted slot shows the sentinel
        const uint64_t kNone = ~0ull;
        int li = 0, ii = n, made = n;
        uint64_t lw0 = nw[0], lw1 = nw[1], iw0 = kNone, iw1 = kNone;
        for (int step = 0; step < n - 1; ++step) {
            int pick[2];
            uint64_t pw[2];
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                if (lw0 != kNone && (iw0 == kNone || lw0 <= iw0)) {
                    pick[r] = li; pw[r] = lw0;
                    ++li;
                    lw0 = lw1;
                    lw1 = li + 1 < n ? nw[li + 1] : kNone;
                } else {
                    pick[r] = ii; pw[r] = iw0;
                    ++ii;
                    iw0 = iw1;
                    iw1 = ii + 1 < made ? nw[ii + 1] : kNone;
                }
            }
            const uint64_t s = pw[0] + pw[1];
            if (s < pw[1] || s == kNone) err = 1;  // the weights of this table sum to 2^64 - 1 or more
            nw[made] = s;
            parent[pick[0]] = made;
            parent[pick[1]] = made;
            if (ii == made) iw0 = s;            // the internal queue was empty: the new node is its head
            else if (ii + 1 == made) iw1 = s;   // it held one node: the new one is second
            ++made;
        }
    }
    __syncthreads();

    if (t < n) {
        int depth = 0;
        if (n == 1) depth = 1;
        for (int p = parent[t]; p >= 0 && depth <= CO3_MAX_CODE_LEN; p = parent[p]) ++depth;
        if (depth > CO3_MAX_CODE_LEN) err = 1;
        else slen[leaf_sym[t]] = (uint32_t)depth;
    }
    __syncthreads();
    const bool bad = err != 0;
    if (bad) {
        slen[t] = 0;
        if (t == 0) atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CODELEN), 1ull);
    }
    __syncthreads();

    const uint32_t L = slen[t];
    if (L) atomicAdd(&cnt[L], 1u);
    __syncthreads();
    if (t == 0) {
        uint64_t code = 0;
        uint32_t o = 0, mx = 0, nlong = 0;
        for (int l = 1; l <= 64; ++l) {
            code = (code + cnt[l - 1]) << 1;
            first[l] = code;
            off[l] = o;
            if (cnt[l]) {
                mx = l;
                if (l > kDecBits) {  // search list for codes longer than the direct table
                    const uint64_t end_code = code + cnt[l];
                    const uint64_t end_la = (l == 64) ? end_code : (end_code << (64 - l));
                    B.long_last[nlong] = end_la - 1;
                    B.long_base[nlong] = o - (uint32_t)code;
                    B.long_len[nlong] = (uint32_t)l;
                    ++nlong;
                }
            }
            o += cnt[l];
        }
        for (uint32_t k = nlong; k < (uint32_t)kLongSlots; ++k) {
            B.long_last[k] = 0; B.long_base[k] = 0; B.long_len[k] = 0;
        }
        B.maxlen = mx;
        B.nactive = bad ? 0 : (uint32_t)n;
        B.nlong = nlong;
    }
    __syncthreads();

    uint64_t code = 0;
    uint32_t fast = kFastSlow << 24;  // a longer code, or none: the coders' general path
    if (L) {
        uint32_t rank = 0;
#pragma unroll 8
        for (int j = 0; j < (int)A; ++j) rank += (uint32_t)((j < t) & (slen[j] == L));
        code = first[L] + rank;
        sorted[off[L] + rank] = (uint32_t)t;
        if (L <= (uint32_t)kFastLen) fast = (L << 24) | (uint32_t)code;
    }
    B.code[t] = code;
    B.fast[t] = fast;
    B.len[t] = (uint8_t)L;
    if (t < 65) { B.first[t] = first[t]; B.count[t] = cnt[t]; B.offset[t] = off[t]; }
    __syncthreads();
    B.sorted[t] = (t < n && !bad) ? (uint8_t)sorted[t] : 0;

    // direct decode table: every kDecBits-bit prefix whose code is at most kDecBits long; the first
    // kDec2Tables prefixes that hold only longer codes (the largest prefixes: canonical codes grow
    // with their length) point to a second-level table over the next kDec2Bits bits
    uint32_t long_prefix0 = kDecEntries;
    for (int l = kDecBits + 1; l <= 64; ++l) {
        if (cnt[l]) { long_prefix0 = (uint32_t)(first[l] >> (l - kDecBits)); break; }
    }
    if (t == 0) B.long_prefix0 = long_prefix0;
    for (int idx = t; idx < kDecEntries; idx += kCbThreads) {
        uint16_t e = 0;
        for (int l = 1; l <= kDecBits; ++l) {
            const uint32_t c = (uint32_t)idx >> (kDecBits - l);
            const uint32_t f = (uint32_t)first[l];
            if (cnt[l] && c >= f && c - f < cnt[l]) {
                e = (uint16_t)((l << 8) | sorted[off[l] + (c - f)]);
                break;
            }
        }
        if (e == 0 && (uint32_t)idx >= long_prefix0 && (uint32_t)idx - long_prefix0 < (uint32_t)kDec2Tables)
            e = (uint16_t)((uint32_t)idx - long_prefix0 + 1);
        B.dec[idx] = e;
    }
    for (int idx = t; idx < (kDec2Tables << kDec2Bits); idx += kCbThreads) {
        const uint32_t wide = ((long_prefix0 + ((uint32_t)idx >> kDec2Bits)) << kDec2Bits) |
                              ((uint32_t)idx & ((1u << kDec2Bits) - 1u));  // kDecBits + kDec2Bits bits
        uint16_t e = 0;
        if ((wide >> kDec2Bits) < (uint32_t)kDecEntries) {
            for (int l = kDecBits + 1; l <= kDecBits + kDec2Bits; ++l) {
                const uint64_t c = wide >> (kDecBits + kDec2Bits - l);
                if (cnt[l] && c >= first[l] && c - first[l] < cnt[l]) {
                    e = (uint16_t)((l << 8) | sorted[off[l] + (uint32_t)(c - first[l])]);
                    break;
                }
            }
        }
        B.dec2[idx] = e;
    }
}

hipError_t launch_build_books(BookDev *books, uint32_t nbooks, uint32_t A, const uint64_t *weights,
                              uint64_t *status, hipStream_t s)
{
    if (nbooks == 0) return hipSuccess;
    ProfScope prof(K_BUILD_BOOKS, s);
    hipLaunchKernelGGL(k_build_books, dim3(nbooks), dim3(kCbThreads), 0, s, books, A, weights, status);
    return hipGetLastError();
}

}  // namespace co3
