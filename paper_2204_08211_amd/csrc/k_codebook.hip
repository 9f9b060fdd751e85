// Huffman code tables built on the device from symbol counts (Sec. IV-A (ii)), one workgroup
// per table, so that an encoder using this round's histogram needs no host round trip.
//
// Same tie rule and canonical form as the host builder: leaves sorted by (weight, symbol),
// internal nodes in creation order, merge the two smallest with leaves first on equal weight.
// The merge runs in rounds that each pair off every node the serial merge would take before any
// node it has yet to create; a table of 256 symbols takes some twenty rounds.
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
    __shared__ uint64_t tmpw[kMaxA];      // a round's nodes in merged order: weight
    __shared__ int tmpid[kMaxA];          // and node index
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

    // The two-queue merge in rounds.  With T the sum of the two lightest nodes alive, every internal node alive and
    // every leaf of weight <= T is taken before any node created from now on (their weights are >= T; on equal
    // weights a leaf goes before an internal node and an older internal node before a newer one).  So the merged
    // order of those nodes — a leaf's rank is its own index plus the number of lighter internal nodes, an internal
    // node's its own plus the number of leaves that are not heavier — pairs off two by two exactly as the serial
    // merge would; an odd one out stays at the head of its queue.  Every thread keeps the queue positions itself;
    // a round has at most A <= 256 nodes, one per thread.
    {
        const uint64_t kNone = ~0ull;
        int li = 0, ii = n, made = n;   // next leaf, next internal node, next node to create
        auto lower_bound = [&](int lo, int hi, uint64_t x) {   // first index in [lo, hi) with nw[index] >= x
            while (lo < hi) { const int mid = (lo + hi) >> 1; if (nw[mid] < x) lo = mid + 1; else hi = mid; }
            return lo;
        };
        auto upper_bound = [&](int lo, int hi, uint64_t x) {   // first index in [lo, hi) with nw[index] > x
            while (lo < hi) { const int mid = (lo + hi) >> 1; if (nw[mid] <= x) lo = mid + 1; else hi = mid; }
            return lo;
        };
        while (n >= 2 && !err && (n - li) + (made - ii) > 1) {   // the same in every thread
            const uint64_t c0 = li < n ? nw[li] : kNone, c1 = li + 1 < n ? nw[li + 1] : kNone;
            const uint64_t c2 = ii < made ? nw[ii] : kNone, c3 = ii + 1 < made ? nw[ii + 1] : kNone;
            // the two lightest of two sorted pairs
            const uint64_t m1 = c0 < c2 ? c0 : c2;
            const uint64_t r1 = c0 < c2 ? c1 : c0, r2 = c0 < c2 ? c2 : c3;
            const uint64_t m2 = r1 < r2 ? r1 : r2;
            const uint64_t T = m1 + m2;
            if (T < m2 || T == kNone) {   // the weights of this table sum to 2^64 - 1 or more
                if (t == 0) err = 1;
                break;
            }
            // leaves of weight <= T: they are sorted, so counting them (thread t looks at leaf li + t) gives the end
            const int bL = __syncthreads_count(li + t < n && nw[li + t] <= T);
            const int lj = li + bL;
            const int bI = made - ii, nb = bL + bI;   // 2 <= nb <= 256: the two lightest are among them
            if (t < nb) {
                int node, r;
                if (t < bL) {
                    node = li + t;
                    r = t + (lower_bound(ii, made, nw[node]) - ii);
                } else {
                    node = ii + (t - bL);
                    r = (t - bL) + (upper_bound(li, lj, nw[node]) - li);
                }
                tmpw[r] = nw[node];
                tmpid[r] = node;
            }
            __syncthreads();
            const int npair = nb >> 1;
            if (t < npair) {
                const uint64_t wa = tmpw[2 * t], wb = tmpw[2 * t + 1];
                const uint64_t sum = wa + wb;
                if (sum < wb || sum == kNone) err = 1;
                nw[made + t] = sum;
                parent[tmpid[2 * t]] = made + t;
                parent[tmpid[2 * t + 1]] = made + t;
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
