// Wavefront-level core of h_Hf (Sec. II-B (iii), Sec. IV-A (ii); Algorithm 1 line 9): the codewords of
// one chunk (4096 symbols) concatenated MSB-first into 32-bit words.  Shared by the coder for stored
// symbols (k_pack.hip) and the single-sweep encoder (k_fused.hip).
//
// A wavefront owns a chunk, lane j owns sub-chunk j (64 symbols, held in 16 registers).
//
// Fast path, two steps:
//   1. every lane concatenates its own codewords, starting at bit 0 of a private LDS row.  No lane
//      needs to know where its bits will land, so no pass over the code lengths comes first: the
//      lane's bit count (the sub-chunk size the decoder's index stores) falls out at the end.
//      Codewords go into a 64-bit shift register two at a time; after each pair at most one 32-bit
//      word is complete and is stored without a branch (a store of the not-yet-complete word is
//      harmless: the slot is written again).  The table entry of a symbol is (length << 24) | code
//      for codes of up to 24 bits.  The length field kFastSlow marks a longer code or none; a pair
//      with such a symbol, or with more than 63 bits pending, ends the fast path for the chunk.
//   2. the wave prefix sum of the lanes' bit counts gives every lane its offset in the chunk; each
//      lane reads its row back into registers, the rows' storage is cleared and becomes the chunk's
//      word window, and every lane ORs its words in, shifted by its offset (neighbouring lanes share
//      a word at most at their two ends).
// General path (a chunk that left the fast path, or a lane whose codewords do not fit its row, i.e. more
// than 12 bits per symbol on average): the symbols go back to LDS, a loop sums the code lengths from the
// full table, and the codewords are appended at their final bit offsets inside a small window, pass by
// pass.  It handles every code length and counts the symbols that have no code.
#pragma once

#include "co3_internal.h"

namespace co3 {

constexpr int kPcRowWords = 24;                          // words of a lane's private row
constexpr int kPcRowStride = kPcRowWords + 1;            // + one slot that takes the stores beyond the row; odd: no bank conflicts
constexpr int kPcRegion = kSubsPerChunk * kPcRowStride;  // 1600 words: staged symbols, then rows, then the chunk's words
constexpr int kPcSymRow = 17;                            // staged symbols: rows of 16 words + 1 pad
constexpr int kPcSymWords = kSubsPerChunk * kPcSymRow;   // 1088
constexpr int kPcWin = kPcRegion - kPcSymWords - 1;      // 511 words: the general path's window, behind the staged symbols
static_assert(kPcWin >= 256, "general window");

__device__ inline void pc_wave_sync_lds()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ inline uint32_t pc_wave_inclusive_scan(uint32_t x, uint32_t lane)
{
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t y = __shfl_up(x, o, 64);
        if ((int)lane >= o) x += y;
    }
    return x;
}

__device__ inline uint32_t pc_wave_max(uint32_t x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t y = __shfl_xor(x, o, 64);
        x = x > y ? x : y;
    }
    return x;
}

// Fast path, step 1.  sym[16]: the lane's 64 symbols, four per word in element order; cnt of them exist
// (the rest of the chunk lies beyond the layer's end).  fast: the code's 32-bit entries in LDS.  region:
// the wavefront's kPcRegion LDS words, free for use (the symbols are in registers); the lane's row starts
// at word lane * kPcRowStride.  Returns true (for the whole wavefront) if every lane's codewords are in its
// row; bits is then the lane's bit count.  On false nothing about the rows holds.
template <bool kFull>
__device__ inline bool pc_pack_rows(const uint32_t (&sym)[kSub / 4], int cnt, const uint32_t *fast, uint32_t *region,
                                    uint32_t lane, uint32_t &bits)
{
    uint64_t acc = 0;                                    // the last 64 bits appended, right-aligned
    uint32_t np = 0;                                     // bits of acc not yet stored: < 32 between pairs
    uint32_t waddr = lane * kPcRowStride;                // row slot the next complete word goes to
    const uint32_t wend = waddr + kPcRowWords;           // the slot behind the row: stores are clamped to it
    bool left = false;
#pragma unroll
    for (int jj = 0; jj < kSub / 4; ++jj) {
#pragma unroll
        for (int q = 0; q < 4; q += 2) {
            const uint32_t s0 = (sym[jj] >> (8 * q)) & 0xffu, s1 = (sym[jj] >> (8 * q + 8)) & 0xffu;
            uint32_t e0 = fast[s0], e1 = fast[s1];
            if (!kFull) {
                e0 = (4 * jj + q < cnt) ? e0 : 0u;          // nothing to append beyond the chunk's end
                e1 = (4 * jj + q + 1 < cnt) ? e1 : 0u;
            }
            const uint32_t L0 = e0 >> 24, L1 = e1 >> 24;
            np += L0 + L1;
            left = left || np > 63u;                        // also every kFastSlow entry (255)
            acc = (acc << (L0 & 63u)) | (e0 & 0x00ffffffu);   // (a kFastSlow entry shifts by 63: harmless, the chunk
            acc = (acc << (L1 & 63u)) | (e1 & 0x00ffffffu);   //  leaves the fast path)
            // store the word the pending bits complete, if they do; otherwise a value the slot outlives
            const uint32_t rest = np & 31u;
            region[waddr < wend ? waddr : wend] = (uint32_t)(acc >> rest);
            waddr += (np >> 5) & 1u;
            np = rest;
        }
    }
    if (__any(left)) return false;
    const uint32_t whole = waddr - lane * kPcRowStride;     // complete words (counted also beyond the row)
    if (np) region[waddr < wend ? waddr : wend] = (uint32_t)(acc << (32u - np));   // left-aligned, zeros below
    bits = whole * 32u + np;
    return !__any(whole + (np ? 1u : 0u) > (uint32_t)kPcRowWords);
}

// Fast path, step 2.  Every lane's row holds its `bits` bits; excl: bits of the lanes before it.  On return
// region[0 .. nwords) holds the chunk's words, nwords = ceil(sum of bits / 32).
__device__ inline void pc_rows_to_window(uint32_t *region, uint32_t lane, uint32_t bits, uint32_t excl, uint32_t nwords)
{
    const uint32_t nw = (bits + 31u) >> 5;                   // <= kPcRowWords
    const uint32_t maxnw = pc_wave_max(nw);                  // wavefront-uniform
    uint32_t r[kPcRowWords];
    const uint32_t *row = region + lane * kPcRowStride;
#pragma unroll
    for (int i = 0; i < kPcRowWords; ++i) {
        r[i] = 0u;
        if ((uint32_t)i < maxnw) r[i] = (uint32_t)i < nw ? row[i] : 0u;
    }
    pc_wave_sync_lds();                                      // all rows are in registers
    for (uint32_t i = lane; i <= nwords; i += 64) region[i] = 0u;
    pc_wave_sync_lds();
    const uint32_t sh = excl & 31u, w0 = excl >> 5;
    uint32_t prev = 0u;
#pragma unroll
    for (int i = 0; i < kPcRowWords; ++i) {
        if ((uint32_t)i < maxnw) {
            const uint32_t out = __builtin_amdgcn_alignbit(prev, r[i], sh);   // ({prev, r[i]} >> sh), low word
            if (out) atomicOr(&region[w0 + (uint32_t)i], out);
            prev = r[i];
        }
    }
    // what the shift pushed out of the lane's last word (rows end in zeros, so prev is that word)
    const uint32_t tail = __builtin_amdgcn_alignbit(prev, 0u, sh);
    if (sh && tail && nw) atomicOr(&region[w0 + nw], tail);
    pc_wave_sync_lds();
}

// General path, first half: the symbols go back to LDS (rows of 16 + 1 words at the front of the region) and
// a loop sums the lane's code lengths from the full table.  Symbols without a code count in `nocode` and
// contribute no bits.
__device__ inline uint32_t pc_general_count(const uint32_t (&sym)[kSub / 4], int cnt, const uint32_t *fast,
                                            const BookDev &book, uint32_t *region, uint32_t lane, uint32_t &nocode)
{
    uint32_t *row = region + lane * kPcSymRow;
#pragma unroll
    for (int jj = 0; jj < kSub / 4; ++jj) row[jj] = sym[jj];
    pc_wave_sync_lds();
    uint32_t total = 0;
    nocode = 0;
    for (int jj = 0; jj < kSub / 4; ++jj) {
        const uint32_t w4 = row[jj];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t s = (w4 >> (8 * q)) & 0xffu;
            const bool in = 4 * jj + q < cnt;
            uint32_t L = in ? (fast[s] >> 24) : 0u;
            if (L == kFastSlow) {
                L = book.len[s];
                nocode += L == 0u ? 1u : 0u;
            }
            total += L;
        }
    }
    return total;
}

// General path, second half: words [wbase, wbase + wn) of the chunk's codewords, wn <= kPcWin, appended at
// their final bit offsets inside win[0 .. wn] = the region behind the staged symbols (lanes OR their words
// in; neighbours share words).  Any code length.
__device__ inline void pc_general_window(int cnt, const uint32_t *fast, const BookDev &book, uint32_t *region, uint32_t lane,
                                         uint32_t excl, uint32_t wbase, uint32_t wn)
{
    const uint32_t *row = region + lane * kPcSymRow;
    uint32_t *win = region + kPcSymWords;
    for (uint32_t i = lane; i <= wn; i += 64) win[i] = 0u;
    pc_wave_sync_lds();
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
    for (int jj = 0; jj < kSub / 4; ++jj) {
        const uint32_t w4 = row[jj];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t s = (w4 >> (8 * q)) & 0xffu;
            const uint32_t e = (4 * jj + q < cnt) ? fast[s] : 0u;
            uint32_t L = e >> 24;
            uint64_t code = e & 0x00ffffffu;
            if (L == kFastSlow) {
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
    if (np && wi < wn) atomicOr(&win[wi], (uint32_t)(acc << (32u - np)));
    pc_wave_sync_lds();
}

}  // namespace co3
