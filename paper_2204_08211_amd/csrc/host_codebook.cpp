// Host construction of one Huffman code table (Sec. IV-A (ii): element-wise Huffman coding of
// the quantized gradient; optimal for a known source, Sec. II-E).
//
// Tie rule: nodes are ordered by (weight, key); a leaf's key is its symbol, an internal node's
// key is A + its creation order; the two smallest are merged.  With the leaves sorted once by
// (weight, symbol) and the internal nodes kept in creation order (their weights never
// decrease), the smallest node is always at the head of one of the two lists, and on equal
// weight the leaf comes first because every leaf key is below every internal key.
#include <algorithm>
#include <cstring>
#include <vector>

#include "co3_internal.h"

namespace co3 {

// Fill every derived table of `b` from b->len[] (lengths) for alphabet size A.
static void finish_tables(BookDev *b, uint32_t A)
{
    std::memset(b->count, 0, sizeof(b->count));
    std::memset(b->first, 0, sizeof(b->first));
    std::memset(b->offset, 0, sizeof(b->offset));
    std::memset(b->code, 0, sizeof(b->code));
    for (uint32_t s = 0; s < (uint32_t)kMaxA; ++s) b->fast[s] = kFastSlow << 24;  // no code: the coders' general path counts it
    std::memset(b->dec, 0, sizeof(b->dec));
    std::memset(b->dec2, 0, sizeof(b->dec2));
    std::memset(b->sorted, 0, sizeof(b->sorted));
    b->maxlen = 0;
    b->nactive = 0;
    for (uint32_t s = 0; s < A; ++s) {
        if (!b->len[s]) continue;
        b->count[b->len[s]]++;
        b->nactive++;
        if (b->len[s] > b->maxlen) b->maxlen = b->len[s];
    }
    // canonical codes: first[L] = (first[L-1] + count[L-1]) << 1
    uint64_t code = 0;
    uint32_t off = 0;
    for (int L = 1; L <= 64; ++L) {
        code = (code + b->count[L - 1]) << 1;
        b->first[L] = code;
        b->offset[L] = off;
        off += b->count[L];
    }
    // search list for codes longer than the direct table
    b->nlong = 0;
    b->long_prefix0 = kDecEntries;
    std::memset(b->long_last, 0, sizeof(b->long_last));
    std::memset(b->long_base, 0, sizeof(b->long_base));
    std::memset(b->long_len, 0, sizeof(b->long_len));
    for (int L = kDecBits + 1; L <= 64; ++L) {
        if (!b->count[L]) continue;
        const uint32_t k = b->nlong++;
        const uint64_t end_code = b->first[L] + b->count[L];                  // 2^L when the code is complete
        const uint64_t end_la = (L == 64) ? end_code : (end_code << (64 - L));  // wraps to 0 then
        b->long_last[k] = end_la - 1;
        b->long_base[k] = b->offset[L] - (uint32_t)b->first[L];
        b->long_len[k] = (uint32_t)L;
    }
    // Prefixes of kDecBits bits under which only longer codes live are the largest ones (canonical
    // codes grow with their length); the first kDec2Tables of them get a second-level table over
    // the next kDec2Bits bits.
    uint32_t long_prefix0 = kDecEntries;
    for (int L = kDecBits + 1; L <= 64; ++L) {
        if (!b->count[L]) continue;
        long_prefix0 = (uint32_t)(b->first[L] >> (L - kDecBits));
        break;
    }
    b->long_prefix0 = long_prefix0;
    for (uint32_t p = long_prefix0; p < (uint32_t)kDecEntries && p - long_prefix0 < (uint32_t)kDec2Tables; ++p)
        b->dec[p] = (uint16_t)(p - long_prefix0 + 1);  // entries of the second-level tables follow with the symbols
    uint32_t next[65];
    std::memset(next, 0, sizeof(next));
    for (uint32_t s = 0; s < A; ++s) {  // ascending symbol within each length
        const int L = b->len[s];
        if (!L) continue;
        const uint32_t rank = next[L]++;
        b->code[s] = b->first[L] + rank;
        b->sorted[b->offset[L] + rank] = (uint8_t)s;
        if (L <= kFastLen) b->fast[s] = ((uint32_t)L << 24) | (uint32_t)b->code[s];
        else b->fast[s] = kFastSlow << 24;
        if (L <= kDecBits) {
            const uint32_t lo = (uint32_t)b->code[s] << (kDecBits - L);
            const uint32_t n = 1u << (kDecBits - L);
            for (uint32_t i = 0; i < n; ++i) b->dec[lo + i] = (uint16_t)((L << 8) | s);
        } else if (L <= kDecBits + kDec2Bits) {
            const uint32_t lo = (uint32_t)b->code[s] << (kDecBits + kDec2Bits - L);
            const uint32_t n = 1u << (kDecBits + kDec2Bits - L);
            for (uint32_t i = 0; i < n; ++i) {
                const uint32_t j = ((lo + i) >> kDec2Bits) - long_prefix0;
                if (j < (uint32_t)kDec2Tables) b->dec2[(j << kDec2Bits) | ((lo + i) & ((1u << kDec2Bits) - 1u))] = (uint16_t)((L << 8) | s);
            }
        }
    }
}

// Huffman code lengths by the two-queue merge (leaves sorted by (weight, symbol), internal nodes in creation
// order, leaves first on equal weight); len must hold A zeros.
static int huffman_lengths_host(const uint64_t *w, uint32_t A, uint8_t *len)
{
    struct Leaf { uint64_t w; uint32_t s; };
    std::vector<Leaf> leaves;
    uint64_t total = 0;
    for (uint32_t s = 0; s < A; ++s) {
        if (!w[s]) continue;
        if (total + w[s] < total || total + w[s] == ~0ull) return CO3_ERR_ARG;
        total += w[s];
        leaves.push_back({w[s], s});
    }
    const int n = (int)leaves.size();
    if (n == 0) return CO3_OK;
    if (n == 1) { len[leaves[0].s] = 1; return CO3_OK; }
    std::sort(leaves.begin(), leaves.end(),
              [](const Leaf &x, const Leaf &y) { return x.w != y.w ? x.w < y.w : x.s < y.s; });
    std::vector<uint64_t> nw(2 * n - 1);
    std::vector<int> parent(2 * n - 1, -1);
    for (int i = 0; i < n; ++i) nw[i] = leaves[i].w;
    int li = 0, ii = n, made = n;
    for (int step = 0; step < n - 1; ++step) {
        int pick[2];
        for (int r = 0; r < 2; ++r) {
            const bool have_leaf = li < n, have_int = ii < made;
            if (have_leaf && (!have_int || nw[li] <= nw[ii])) pick[r] = li++;
            else pick[r] = ii++;
        }
        nw[made] = nw[pick[0]] + nw[pick[1]];
        parent[pick[0]] = made;
        parent[pick[1]] = made;
        ++made;
    }
    for (int i = 0; i < n; ++i) {
        int depth = 0;
        for (int p = parent[i]; p >= 0; p = parent[p]) ++depth;
        if (depth > CO3_MAX_CODE_LEN) return CO3_ERR_CODELEN;
        len[leaves[i].s] = (uint8_t)depth;
    }
    return CO3_OK;
}

int build_wide_host(const uint64_t *w, uint32_t A, BookWide *b)
{
    std::memset(b, 0, sizeof(*b));
    int rc = huffman_lengths_host(w, A, b->len);
    if (rc != CO3_OK) { std::memset(b, 0, sizeof(*b)); return rc; }
    for (uint32_t s = 0; s < A; ++s) {
        if (!b->len[s]) continue;
        b->count[b->len[s]]++;
        b->nactive++;
        if (b->len[s] > b->maxlen) b->maxlen = b->len[s];
    }
    uint64_t code = 0;
    uint32_t off = 0;
    for (int L = 1; L <= 64; ++L) {   // canonical codes: first[L] = (first[L-1] + count[L-1]) << 1
        code = (code + b->count[L - 1]) << 1;
        b->first[L] = code;
        b->offset[L] = off;
        off += b->count[L];
    }
    uint32_t next[65];
    std::memset(next, 0, sizeof(next));
    for (uint32_t s = 0; s < A; ++s) {  // ascending symbol within each length
        const int L = b->len[s];
        if (!L) continue;
        const uint32_t rank = next[L]++;
        b->code[s] = b->first[L] + rank;
        b->sorted[b->offset[L] + rank] = (uint16_t)s;
        if (L <= kWideDecBits) {
            const uint32_t lo = (uint32_t)b->code[s] << (kWideDecBits - L);
            for (uint32_t i = 0; i < (1u << (kWideDecBits - L)); ++i) b->dec[lo + i] = (uint16_t)((L << 12) | s);
        }
    }
    // second-level tables under the first prefixes that hold only longer codes
    b->long_prefix0 = 1u << kWideDecBits;
    for (int L = kWideDecBits + 1; L <= 64; ++L)
        if (b->count[L]) { b->long_prefix0 = (uint32_t)(b->first[L] >> (L - kWideDecBits)); break; }
    for (uint32_t s = 0; s < A; ++s) {
        const int L = b->len[s];
        if (L <= kWideDecBits || L > kWideDecBits + kWideDec2Bits) continue;
        const uint32_t span = kWideDecBits + kWideDec2Bits;
        const uint32_t lo = (uint32_t)b->code[s] << (span - L);   // the code followed by zeros, span bits
        const uint32_t tab = (lo >> kWideDec2Bits) - b->long_prefix0;
        if (tab >= (uint32_t)kWideDec2Tables) continue;
        for (uint32_t i = 0; i < (1u << (span - L)); ++i)
            b->dec2[(tab << kWideDec2Bits) | ((lo + i) & ((1u << kWideDec2Bits) - 1u))] =
                (uint16_t)(((L - kWideDecBits) << 12) | s);
    }
    return CO3_OK;
}

int build_book_host(const uint64_t *w, uint32_t A, BookDev *b)
{
    std::memset(b, 0, sizeof(*b));
    struct Leaf { uint64_t w; uint32_t s; };
    std::vector<Leaf> leaves;
    uint64_t total = 0;
    for (uint32_t s = 0; s < A; ++s) {
        if (!w[s]) continue;
        if (total + w[s] < total || total + w[s] == ~0ull) return CO3_ERR_ARG;
        total += w[s];
        leaves.push_back({w[s], s});
    }
    const int n = (int)leaves.size();
    if (n == 0) { finish_tables(b, A); return CO3_OK; }
    if (n == 1) { b->len[leaves[0].s] = 1; finish_tables(b, A); return CO3_OK; }
    std::sort(leaves.begin(), leaves.end(),
              [](const Leaf &x, const Leaf &y) { return x.w != y.w ? x.w < y.w : x.s < y.s; });
    // nodes 0..n-1: sorted leaves; n..2n-2: internal nodes in creation order
    std::vector<uint64_t> nw(2 * n - 1);
    std::vector<int> parent(2 * n - 1, -1);
    for (int i = 0; i < n; ++i) nw[i] = leaves[i].w;
    int li = 0, ii = n, made = n;
    for (int step = 0; step < n - 1; ++step) {
        int pick[2];
        for (int r = 0; r < 2; ++r) {
            const bool have_leaf = li < n, have_int = ii < made;
            if (have_leaf && (!have_int || nw[li] <= nw[ii])) pick[r] = li++;
            else pick[r] = ii++;
        }
        nw[made] = nw[pick[0]] + nw[pick[1]];
        parent[pick[0]] = made;
        parent[pick[1]] = made;
        ++made;
    }
    for (int i = 0; i < n; ++i) {
        int depth = 0;
        for (int p = parent[i]; p >= 0; p = parent[p]) ++depth;
        if (depth > CO3_MAX_CODE_LEN) return CO3_ERR_CODELEN;
        b->len[leaves[i].s] = (uint8_t)depth;
    }
    finish_tables(b, A);
    return CO3_OK;
}

}  // namespace co3
