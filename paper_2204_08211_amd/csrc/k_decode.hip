// PS side (Sec. II-B (iv); Algorithm 1 lines 13-14): invert h_Hf for every user's stream and
// form (1/U) sum_u ghat^(u), eq. (aggregate hat) without the learning rate.
//
// A wavefront decodes one chunk of one user.  It first copies the chunk's words from HBM into
// LDS with coalesced loads; then lane j decodes sub-chunk j (64 elements), whose start is the
// prefix sum of the sub-chunk bit counts.  Codes of up to kDecBits bits are resolved by one LDS
// table lookup, a little longer ones by a second-level table, the rest by a search over the
// canonical code's length boundaries.  co3_decode and the average for few users stage the decoded
// symbols in LDS so that global stores (and the sum over users) are coalesced; the average for
// many users adds every value to fp64 sums in LDS as it is decoded.  A chunk whose words do not
// fit the LDS window is decoded straight from global memory (same code, slower).
//
// The work moves about b/8 + 4/U bytes per element and is bound by how many sub-chunk streams a
// CU keeps in flight (each needs its chunk's words in LDS), not by HBM.
#include <cstddef>
#include <cstdlib>

#include "co3_internal.h"
#include "quantize_math.h"

namespace co3 {

constexpr int kStageStride = 17;                            // words per staged sub-chunk row (16 + 1 pad)
constexpr int kStageWords = kSubsPerChunk * kStageStride;   // one chunk of one user
constexpr int kPayloadWords = 1088;                         // a chunk of up to 8.5 bit/element is decoded from LDS
constexpr int kPayloadPerLane = kPayloadWords / 64;
// Allocated words of the LDS window.  A lane starts at most at word kPayloadWords, holds two words
// and takes at most one more per symbol, so its reads end below kPayloadWords + 2 + kSub.
constexpr int kPayloadAlloc = kPayloadWords + 2 + kSub + 6;

// Decode tables of one code in LDS.
struct DecLds {
    uint16_t dec[kDecEntries];
    uint16_t dec2[kDec2Tables << kDec2Bits];
    uint64_t long_last[kLongSlots];
    uint32_t long_base[kLongSlots];
    uint32_t long_len[kLongSlots];
    uint8_t sorted[kMaxA];
    uint32_t nlong;
    uint32_t long_prefix0;
};
static_assert(offsetof(DecLds, dec) == 0 && offsetof(DecLds, dec2) == sizeof(uint16_t) * kDecEntries,
              "the direct table comes first and the second-level tables directly follow it");

__device__ inline void load_dec_tables(DecLds *T, const BookDev &book, uint32_t t, uint32_t nthreads)
{
    for (uint32_t i = t; i < kDecEntries / 2; i += nthreads)
        reinterpret_cast<uint32_t *>(T->dec)[i] = reinterpret_cast<const uint32_t *>(book.dec)[i];
    for (uint32_t i = t; i < (uint32_t)((kDec2Tables << kDec2Bits) / 2); i += nthreads)
        reinterpret_cast<uint32_t *>(T->dec2)[i] = reinterpret_cast<const uint32_t *>(book.dec2)[i];
    for (uint32_t i = t; i < (uint32_t)kLongSlots; i += nthreads) {
        T->long_last[i] = book.long_last[i];
        T->long_base[i] = book.long_base[i];
        T->long_len[i] = book.long_len[i];
    }
    for (uint32_t i = t; i < kMaxA / 4; i += nthreads)
        reinterpret_cast<uint32_t *>(T->sorted)[i] = reinterpret_cast<const uint32_t *>(book.sorted)[i];
    if (t == 0) { T->nlong = book.nlong; T->long_prefix0 = book.long_prefix0; }
}

// The PS average with tables shared by the users reads one table: per prefix (direct table, then the second-level
// tables, as one array) the code length in bits 16.. and, below, the top 16 bits of the fp32 pattern of the
// symbol's value at exponent bias 0 (sign, exponent and 7 mantissa bits: a representative of a format of up to
// 8 bits has at most 5).  The value for a user is that number times 2^-bias (exact), times the user's scale.
// 0: no codeword of up to kDecBits + kDec2Bits bits under this prefix.
constexpr int kValEntries = kDecEntries + (kDec2Tables << kDec2Bits);
// What the rare decode path needs of a code.
struct LongLds {
    uint64_t long_last[kLongSlots];
    uint32_t long_base[kLongSlots];
    uint32_t long_len[kLongSlots];
    uint8_t sorted[kMaxA];
    uint32_t nlong;
    uint32_t long_prefix0;
};

__device__ inline void load_value_tables(LongLds *T, uint32_t *val, const BookDev &book, int E, int M, uint32_t t,
                                         uint32_t nthreads)
{
    for (uint32_t i = t; i < (uint32_t)kValEntries; i += nthreads) {
        const uint32_t e = i < (uint32_t)kDecEntries ? book.dec[i] : book.dec2[i - kDecEntries];
        const uint32_t L = e >> 8;
        val[i] = L ? (L << 16) | (symbol_value_bits(e & 0xffu, E, M, 0) >> 16) : 0u;
    }
    for (uint32_t i = t; i < (uint32_t)kLongSlots; i += nthreads) {
        T->long_last[i] = book.long_last[i];
        T->long_base[i] = book.long_base[i];
        T->long_len[i] = book.long_len[i];
    }
    for (uint32_t i = t; i < kMaxA / 4; i += nthreads)
        reinterpret_cast<uint32_t *>(T->sorted)[i] = reinterpret_cast<const uint32_t *>(book.sorted)[i];
    if (t == 0) { T->nlong = book.nlong; T->long_prefix0 = book.long_prefix0; }
}

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

// Word sources of the decoder: index 0 is the chunk's first word.  A well-formed stream never
// consumes bits beyond its chunk; what a read beyond the end returns only has to be harmless.
// word(i): any i.  next(i): the reader's sequential fetch, i below seek_limit + 2 + kSub.
struct LdsWords {
    const uint32_t *base;   // kPayloadAlloc allocated words; the chunk's words in front
    static constexpr uint32_t seek_limit = kPayloadWords;
    __device__ inline uint32_t word(uint32_t i) const
    {
        return base[i < (uint32_t)(kPayloadAlloc - 1) ? i : (uint32_t)(kPayloadAlloc - 1)];
    }
    __device__ inline uint32_t next(uint32_t i) const { return base[i]; }
};
struct GlobalWords {
    const uint32_t *base;   // chunk's first word in the user's stream
    uint64_t n;             // words of the chunk
    static constexpr uint32_t seek_limit = 0xffffff00u;
    __device__ inline uint32_t word(uint32_t i) const { return i < n ? base[i] : 0u; }
    __device__ inline uint32_t next(uint32_t i) const { return word(i); }
};

// (length << 8) | symbol of the code longer than kDecBits that starts at bit `pos` of the chunk,
// 0 if none matches.  Left-aligned canonical codes grow with their length, so the code's length
// is the first listed one whose last code is not below the window.
template <class Src, class Tab>
__device__ __noinline__ uint32_t long_code(Src src, const Tab *T, uint32_t pos)
{
    const uint32_t i0 = pos >> 5, s0 = pos & 31u;
    uint64_t full = (((uint64_t)src.word(i0) << 32) | src.word(i0 + 1)) << s0;
    if (s0) full |= (uint64_t)(src.word(i0 + 2) >> (32u - s0));
    const uint32_t n = T->nlong;
    for (uint32_t k = 0; k < n; ++k) {
        if (full <= T->long_last[k]) {
            const uint32_t L = T->long_len[k];
            const uint32_t idx = (uint32_t)(full >> (64u - L)) + T->long_base[k];
            return (L << 8) | T->sorted[idx & (kMaxA - 1)];
        }
    }
    return 0u;
}

// Sequential bit reader of one lane: two consecutive words w0, w1 of the stream, of which the first c bits of
// w0 (1 <= c <= 32) are consumed; kept is k = 32 - c, so that the next 32 bits are one v_alignbit of (w0, w1) by
// k.  Consuming at most 32 bits moves on by at most one word.
template <class Src>
struct Reader {
    Src src;
    uint32_t w0, w1;   // word with the next bit (or, with k = 0, the word before it), following word
    uint32_t k;        // 32 - (consumed bits of w0), 0..31
    uint32_t wi;       // index of the word after w1
    __device__ inline void seek(uint32_t pos)
    {
        uint32_t i = pos >> 5;
        i = i < Src::seek_limit ? i : Src::seek_limit;
        const uint32_t sh = pos & 31u;
        w0 = sh ? src.word(i) : 0u;        // at a word boundary w0 counts as consumed entirely
        w1 = src.word(sh ? i + 1u : i);
        wi = sh ? i + 2u : i + 1u;
        k = (32u - sh) & 31u;
    }
    __device__ inline uint32_t pos() const { return (wi - 2u) * 32u + (32u - k); }
    // the next 32 bits
    __device__ inline uint32_t window32() const { return __builtin_amdgcn_alignbit(w0, w1, k); }
    // the next 64 bits, `nextw` being word wi
    __device__ inline uint64_t window64(uint32_t nextw) const
    {
        return ((uint64_t)__builtin_amdgcn_alignbit(w0, w1, k) << 32) | __builtin_amdgcn_alignbit(w1, nextw, k);
    }
    // L <= 32 bits consumed; `nextw` is word wi
    __device__ inline void advance(uint32_t L, uint32_t nextw)
    {
        const int32_t t = (int32_t)k - (int32_t)L;
        const bool take = t < 0;
        k = (uint32_t)t & 31u;
        w0 = take ? w1 : w0;
        w1 = take ? nextw : w1;
        wi += take ? 1u : 0u;
    }
};

// The rare part of decode_symbol, for the lanes whose look-up found no codeword (L == 0 on entry: a code longer
// than kDecBits + kDec2Bits bits, or a stream that is not one): the window is compared with the left-aligned
// last code of every longer length that occurs (they grow with the length).  Lengths up to 32 are consumed by
// the caller; longer ones take the exact path, which repositions the reader itself and leaves L = 0.
template <class Src, class Tab>
__device__ inline void decode_symbol_long(Reader<Src> &r, const Tab *T, uint64_t win, uint32_t &L, uint32_t &s, bool &bad)
{
    if (L != 0u) return;
    const uint32_t n = T->nlong;
    uint32_t k = 0;
    while (k < n && win > T->long_last[k]) ++k;
    if (k < n) {
        L = T->long_len[k];
        if (L <= 32u) s = T->sorted[((uint32_t)(win >> (64u - L)) + T->long_base[k]) & (kMaxA - 1)];
    }
    if (L == 0u || L > 32u) {
        const uint32_t pos = r.pos();
        const uint32_t code = long_code(r.src, T, pos);  // exact 64-bit window
        uint32_t len = code >> 8;
        s = code & 0xffu;
        if (len == 0u) { bad = true; len = 1u; }
        r.seek(pos + len);
        L = 0u;                                          // the reader stands behind the code already
    }
}

// One symbol; `bad` is set if nothing matched.  The common case is one look-up and a branch-free advance.  The
// look-up covers codes of up to kDecBits + kDec2Bits bits: the next kDecBits bits index the direct table, unless
// they are one of the first kDec2Tables prefixes under which only longer codes live (p0 = the first such prefix;
// canonical codes grow with their length, so these are the largest prefixes) - then kDec2Bits more bits index that
// prefix's second-level table, which lies directly behind the direct table.  The branch to the rare part is taken
// by the whole wavefront or not at all.  Returned is the symbol in bits 0..7; the bits above are not defined (the
// table's entry is passed on as it is).  While the LDS reads of this symbol are in flight the sink may have one of
// its own for the symbol before (`pend`, element j): Sink::fetch requests it, Sink::commit uses it, and the
// wavefront waits once for all of them.
template <bool kCommit, class Src, class Sink>
__device__ inline uint32_t decode_symbol(Reader<Src> &r, const DecLds *T, uint32_t p0, bool &bad, Sink &sink, int j,
                                         uint32_t pend)
{
    const uint32_t win = r.window32();
    const uint32_t i1 = win >> (32 - kDecBits);
    const uint32_t i2 = (uint32_t)kDecEntries + (win >> (32 - kDecBits - kDec2Bits)) - (p0 << kDec2Bits);
    const uint32_t idx = (i1 - p0 < (uint32_t)kDec2Tables) ? i2 : i1;   // unsigned: false below p0
    uint32_t nextw = r.src.next(r.wi);                       // all LDS reads are requested
    uint32_t e = reinterpret_cast<const uint16_t *>(T)[idx]; // dec[] and, behind it, dec2[]; before any result is needed
    uint32_t tok = kCommit ? sink.fetch(pend) : 0u;
    asm volatile("" : "+v"(nextw), "+v"(e), "+v"(tok));
    if (kCommit) sink.commit(j, pend, tok);
    uint32_t L = e >> 8, s = e;
    if (__builtin_expect(__any(L == 0u), 0)) {
        decode_symbol_long(r, T, r.window64(nextw), L, s, bad);
        asm volatile("" : "+v"(L), "+v"(s));   // the rare part waits for its own LDS reads: none is left pending for the common path
    }
    r.advance(L, nextw);
    return s;
}

// Where a lane's decoded symbols go (bits above bit 7 of a symbol are to be ignored).
// StageSink: four per word into an LDS row (co3_decode: coalesced stores of symbols and values follow).
struct StageSink {
    uint32_t *row;
    uint32_t packed;
    __device__ inline uint32_t fetch(uint32_t) const { return 0u; }
    __device__ inline void commit(int j, uint32_t s, uint32_t)
    {
        packed |= (s & 0xffu) << (8 * (j & 3));
        if ((j & 3) == 3) { row[j >> 2] = packed; packed = 0; }
    }
    __device__ inline void finish(int cnt) { if (cnt & 3) row[cnt >> 2] = packed; }
};
// AccSink: the symbol's value is added to the element's fp64 accumulator in LDS (co3_ps_aggregate).  The value
// is the magnitude's entry in the user's table of fp32 patterns with the symbol's sign bit moved to bit 31.
struct AccSink {
    double *row;            // the lane's 64 accumulators
    const uint32_t *mag;
    uint32_t mag_mask, sign_up;
    __device__ inline uint32_t fetch(uint32_t s) const { return mag[s & mag_mask]; }
    __device__ inline void commit(int j, uint32_t s, uint32_t m)
    {
        const uint32_t bits = m | ((s << sign_up) & 0x80000000u);
        __hip_atomic_fetch_add(&row[j], (double)__uint_as_float(bits), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    __device__ inline void finish(int) {}
};

// Decode `cnt` (<= 64) symbols of one sub-chunk starting `p0` bits into the chunk and hand them to the sink.
// Returns the number of bits consumed, or ~0u if a prefix matched no codeword.
template <class Src, class Sink>
__device__ inline uint32_t decode_subchunk(Src src, uint32_t p0, int cnt, const DecLds *T, Sink sink)
{
    Reader<Src> r;
    r.src = src;
    r.seek(p0);
    bool bad = false;
    const uint32_t lp0 = T->long_prefix0;   // read once: the sinks' LDS traffic would make the compiler reload it
    if (cnt == kSub) {
        // the sink's work for symbol j runs beside the decoding of symbol j + 1
        uint32_t pend = decode_symbol<false>(r, T, lp0, bad, sink, 0, 0u);
        for (int jj = 0; jj < kSub / 4 - 1; ++jj) {
#pragma unroll
            for (int b = 0; b < 4; ++b) pend = decode_symbol<true>(r, T, lp0, bad, sink, 4 * jj + b, pend);
        }
#pragma unroll
        for (int b = 0; b < 3; ++b) pend = decode_symbol<true>(r, T, lp0, bad, sink, kSub - 4 + b, pend);
        sink.commit(kSub - 1, pend, sink.fetch(pend));
    } else {
        for (int j = 0; j < cnt; ++j) {
            const uint32_t sy = decode_symbol<false>(r, T, lp0, bad, sink, 0, 0u);
            sink.commit(j, sy, sink.fetch(sy));
        }
        sink.finish(cnt);
    }
    return bad ? ~0u : r.pos() - p0;
}

// The PS average's decoder for tables shared by the users: one look-up per symbol gives its length and its value
// (see kValEntries), which goes straight to the element's fp64 sum in LDS.  nbias = -bias of the user and layer.
template <class Src>
__device__ inline uint32_t decode_subchunk_acc(Src src, uint32_t p0, int cnt, const LongLds *T, const uint32_t *val,
                                               int E, int M, int nbias, float inv_gain, double *row)
{
    Reader<Src> r;
    r.src = src;
    r.seek(p0);
    bool bad = false;
    const uint32_t lp0 = T->long_prefix0;   // read once: the LDS atomics would make the compiler reload it
    auto one = [&](int j) {
        const uint32_t win = r.window32();
        const uint32_t i1 = win >> (32 - kDecBits);
        const uint32_t i2 = (uint32_t)kDecEntries + (win >> (32 - kDecBits - kDec2Bits)) - (lp0 << kDec2Bits);
        const uint32_t idx = (i1 - lp0 < (uint32_t)kDec2Tables) ? i2 : i1;   // unsigned: false below lp0
        uint32_t nextw = r.src.next(r.wi);
        uint32_t e = val[idx];
        asm volatile("" : "+v"(nextw), "+v"(e));
        uint32_t L = e >> 16;
        float v = __fmul_rn(ldexpf(__uint_as_float(e << 16), nbias), inv_gain);
        if (__builtin_expect(__any(L == 0u), 0)) {
            const bool mine = L == 0u;
            uint32_t sy = 0;
            decode_symbol_long(r, T, r.window64(nextw), L, sy, bad);
            if (mine) v = __fmul_rn(__uint_as_float(symbol_value_bits(sy & 0xffu, E, M, -nbias)), inv_gain);
            asm volatile("" : "+v"(L), "+v"(v));   // the rare part waits for its own LDS reads
        }
        __hip_atomic_fetch_add(&row[j], (double)v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        r.advance(L, nextw);
    };
    if (cnt == kSub) {
        for (int jj = 0; jj < kSub / 4; ++jj) {
#pragma unroll
            for (int b = 0; b < 4; ++b) one(4 * jj + b);
        }
    } else {
        for (int j = 0; j < cnt; ++j) one(j);
    }
    return bad ? ~0u : r.pos() - p0;
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

// What a wavefront needs to know about chunk c of user u before it can decode it.
struct ChunkIndex {
    const uint32_t *w;   // chunk's first word
    uint32_t nw;         // its words (0 if the index is malformed)
    uint32_t sb;         // this lane's sub-chunk bit count
    bool ok;             // 32-bit aligned, ordered, inside the buffer
    bool in_lds;         // fits the LDS window
};

__device__ inline ChunkIndex read_index(const Layout &lay, uint64_t c, uint32_t u, const uint32_t *__restrict__ words,
                                        uint64_t words_stride, const uint64_t *__restrict__ chunk_offset,
                                        const uint16_t *__restrict__ sub_bits)
{
    ChunkIndex ix;
    const uint32_t lane = threadIdx.x & 63;
    const uint64_t off = chunk_offset[(uint64_t)u * (lay.nchunks + 1) + c];
    const uint64_t end = chunk_offset[(uint64_t)u * (lay.nchunks + 1) + c + 1];
    ix.sb = sub_bits[((uint64_t)u * lay.nchunks + c) * kSubsPerChunk + lane];
    ix.ok = !(off & 31u) && end >= off && (end >> 5) <= words_stride &&
            ((end - off) >> 5) <= (uint64_t)kChunk * CO3_MAX_CODE_LEN / 32;
    ix.nw = ix.ok ? (uint32_t)((end - off) >> 5) : 0u;
    ix.w = words + (uint64_t)u * words_stride + (ix.ok ? (off >> 5) : 0);
    ix.in_lds = ix.nw <= (uint32_t)kPayloadWords;
    return ix;
}

// The chunk's words as the wavefront requests them from HBM: word lane + 64 k in tmp[k] (zero beyond the chunk, and
// nothing is requested for a chunk that does not fit the LDS window).
__device__ inline void payload_request(const ChunkIndex &ix, uint32_t (&tmp)[kPayloadPerLane])
{
    const uint32_t lane = threadIdx.x & 63;
#pragma unroll
    for (int k = 0; k < kPayloadPerLane; ++k) {
        const uint32_t i = lane + 64u * k;
        tmp[k] = (ix.in_lds && i < ix.nw) ? ix.w[i] : 0u;
    }
}

// One wavefront: the requested words go to s_pay (if the chunk fits), the chunk is decoded into the lanes' sinks.
// Every read of the stream stays inside the chunk's words.  Inconsistent sub-chunks are counted in
// status[CO3_STAT_CORRUPT].  Contains wave-level synchronisation only.
template <class Sink>
__device__ inline void decode_requested_chunk(const ChunkGeom &g, const ChunkIndex &ix, const DecLds *T, uint32_t *s_pay,
                                              const uint32_t (&tmp)[kPayloadPerLane], Sink sink, uint64_t *status)
{
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t p0 = wave_exclusive_scan_u32(ix.sb);
    const int first_elem = (int)lane * kSub;
    const int cnt = (int)g.n - first_elem < 0 ? 0 : ((int)g.n - first_elem > kSub ? kSub : (int)g.n - first_elem);
    uint32_t used = 0;
    if (ix.in_lds) {
#pragma unroll
        for (int k = 0; k < kPayloadPerLane; ++k) {
            const uint32_t i = lane + 64u * k;
            if (i < ix.nw) s_pay[i] = tmp[k];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        if (cnt > 0) used = decode_subchunk(LdsWords{s_pay}, p0, cnt, T, sink);
    } else if (cnt > 0) {
        used = decode_subchunk(GlobalWords{ix.w, ix.nw}, p0, cnt, T, sink);
    }
    if (used != ix.sb || !ix.ok)
        atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CORRUPT), 1ull);
}

// The two in one go: all loads first, then all LDS stores, one memory latency for the whole chunk.
template <class Sink>
__device__ inline void decode_user_chunk(const ChunkGeom &g, const ChunkIndex &ix, const DecLds *T,
                                         uint32_t *s_pay, Sink sink, uint64_t *status)
{
    uint32_t tmp[kPayloadPerLane];
    payload_request(ix, tmp);
    decode_requested_chunk(g, ix, T, s_pay, tmp, sink, status);
}

// co3_decode: a workgroup takes one chunk of kDecWaves consecutive users, a wavefront per user, so
// that the users share one copy of the code's tables in LDS (with per-user tables every wavefront
// loads its own).  After decoding, every wavefront writes its own chunk out: no workgroup barrier
// follows the one that publishes the tables.
constexpr int kDecWaves = 8;
__global__ __launch_bounds__(64 * kDecWaves) void k_decode(Layout lay, const uint32_t *__restrict__ words,
                                                           uint64_t words_stride,
                                                           const uint64_t *__restrict__ chunk_offset,
                                                           const uint16_t *__restrict__ sub_bits,
                                                           const BookDev *__restrict__ books, uint8_t *__restrict__ sym,
                                                           uint64_t sym_stride, float *__restrict__ q, uint64_t q_stride,
                                                           uint64_t *__restrict__ status)
{
    extern __shared__ uint64_t smem64[];
    DecLds *s_tab = reinterpret_cast<DecLds *>(smem64);   // [per-user books ? kDecWaves : 1]
    const uint32_t ntab = lay.per_user_books ? kDecWaves : 1;
    uint32_t *s_stage_all = reinterpret_cast<uint32_t *>(s_tab + ntab);    // [kDecWaves][kStageWords]
    uint32_t *s_pay_all = s_stage_all + kDecWaves * kStageWords;           // [kDecWaves][kPayloadAlloc]
    const uint32_t t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const uint64_t c = blockIdx.x;
    const uint32_t u = blockIdx.y * kDecWaves + wave;
    const bool active = u < lay.U;
    const ChunkGeom g = chunk_geom(lay, c);
    ChunkIndex ix;
    if (active) ix = read_index(lay, c, u, words, words_stride, chunk_offset, sub_bits);
    const DecLds *my_tab = s_tab;
    if (lay.per_user_books) {
        my_tab = s_tab + wave;
        if (active) load_dec_tables(s_tab + wave, books[u * lay.books_per_user + (uint32_t)g.book], lane, 64);
    } else {
        load_dec_tables(s_tab, books[(uint32_t)g.book], t, 64 * kDecWaves);
    }
    __syncthreads();
    if (!active) return;  // whole wavefront; wavefront-level synchronisation only from here on
    uint32_t *s_stage = s_stage_all + wave * kStageWords;
    decode_user_chunk(g, ix, my_tab, s_pay_all + wave * kPayloadAlloc, StageSink{s_stage + lane * kStageStride, 0u}, status);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
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
        const float inv_gain = lay.gain[2 * ((uint64_t)u * lay.nseg + g.seg) + 1];   // 1 unless the plan carries a scale
        float *dst = q + (uint64_t)u * q_stride + g.e0;
        for (uint32_t e = lane; e < g.n; e += 64) {
            const uint32_t s = stage_b[(e >> 6) * (kStageStride * 4) + (e & 63u)];
            dst[e] = __fmul_rn(__uint_as_float(symbol_value_bits(s, lay.E, lay.M, bias)), inv_gain);
        }
    }
}

constexpr int kMagEntries = kMaxA / 2;  // magnitude codes of a symbol alphabet (the sign bit is on top)
constexpr int kAccStride = kSub + 1;    // a lane's 64 accumulators + 1 pad: lanes hit different banks
constexpr int kAccWords = kSubsPerChunk * kAccStride;

// The PS average for few users (U <= 4): W = U wavefronts decode the users' chunks into staged symbol rows (as
// co3_decode does), then every thread sums its elements over the users in fp64, in user order.  It needs no
// accumulators in LDS, so that a workgroup of few wavefronts still leaves room for several per CU; with many users
// k_aggregate below, whose footprint does not grow with W, keeps more wavefronts in flight.
template <int W>
__global__ __launch_bounds__(64 * W) void k_aggregate_staged(Layout lay, const uint32_t *__restrict__ words,
                                                      uint64_t words_stride,
                                                      const uint64_t *__restrict__ chunk_offset,
                                                      const uint16_t *__restrict__ sub_bits,
                                                      const BookDev *__restrict__ books, float *__restrict__ out,
                                                      float *__restrict__ model, float eta,
                                                      uint64_t *__restrict__ status)
{
    extern __shared__ uint64_t smem64[];
    DecLds *s_tab = reinterpret_cast<DecLds *>(smem64);   // [per-user books ? W : 1]
    const uint32_t ntab = lay.per_user_books ? W : 1;
    uint32_t *s_mag = reinterpret_cast<uint32_t *>(s_tab + ntab);          // [W][kMagEntries] fp32 patterns
    uint32_t *s_stage = s_mag + W * kMagEntries;                           // [W][kStageWords]
    uint32_t *s_pay = s_stage + W * kStageWords;                           // [W][kPayloadAlloc]
    constexpr int T = 64 * W;
    constexpr int G = (kChunk / 4) / T;  // 4-element groups per thread
    const uint32_t t = threadIdx.x, wave = t >> 6;
    const uint64_t c = blockIdx.x;
    const ChunkGeom g = chunk_geom(lay, c);
    const uint32_t sign_shift = (uint32_t)(lay.E + lay.M);
    const uint32_t mag_mask = (1u << sign_shift) - 1u;
    const uint32_t sign_up = 31u - sign_shift;

    double acc[G][4];
#pragma unroll
    for (int i = 0; i < G; ++i)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[i][b] = 0.0;

    for (uint32_t u0 = 0; u0 < lay.U; u0 += W) {
        const uint32_t u = u0 + wave;
        const bool active = u < lay.U;
        ChunkIndex ix;
        if (active) ix = read_index(lay, c, u, words, words_stride, chunk_offset, sub_bits);
        const DecLds *my_tab = s_tab;
        if (lay.per_user_books) {
            my_tab = s_tab + wave;
            if (active) load_dec_tables(s_tab + wave, books[u * lay.books_per_user + (uint32_t)g.book], t & 63u, 64);
        } else if (u0 == 0) {
            load_dec_tables(s_tab, books[(uint32_t)g.book], t, T);
        }
        for (uint32_t i = t; i < (uint32_t)(W * kMagEntries); i += T) {
            const uint32_t uu = i / kMagEntries, k = i % kMagEntries;
            if (u0 + uu < lay.U && k <= mag_mask) {
                const uint64_t pair = (uint64_t)(u0 + uu) * lay.nseg + g.seg;
                s_mag[i] = __float_as_uint(__fmul_rn(__uint_as_float(symbol_value_bits(k, lay.E, lay.M, lay.bias[pair])),
                                                     lay.gain[2 * pair + 1]));   // inv_gain: 1 unless the plan carries a scale
            }
        }
        __syncthreads();
        if (active)
            decode_user_chunk(g, ix, my_tab, s_pay + wave * kPayloadAlloc,
                              StageSink{s_stage + wave * kStageWords + (t & 63u) * kStageStride, 0u}, status);
        __syncthreads();
        const uint32_t nu = (lay.U - u0 < (uint32_t)W) ? lay.U - u0 : (uint32_t)W;
        for (uint32_t uu = 0; uu < nu; ++uu) {
            const uint32_t *mag = s_mag + uu * kMagEntries;
            const uint32_t *st = s_stage + uu * kStageWords;
#pragma unroll
            for (int i = 0; i < G; ++i) {
                const uint32_t e4 = t + (uint32_t)i * T;  // group of elements 4*e4 .. 4*e4+3
                const uint32_t wv = st[(e4 >> 4) * kStageStride + (e4 & 15u)];
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint32_t s = (wv >> (8 * b)) & 0xffu;
                    const uint32_t bits = mag[s & mag_mask] | ((s << sign_up) & 0x80000000u);
                    acc[i][b] += (double)__uint_as_float(bits);
                }
            }
        }
        __syncthreads();
    }
    // average, and with `model` the PS update w - eta * average (eq. (aggregate hat), Algorithm 1
    // line 14): products and difference in fp64, one rounding
    const double inv_u = 1.0 / (double)lay.U;
    const double eta64 = (double)eta;
    const uintptr_t out_addr = out ? reinterpret_cast<uintptr_t>(out + g.e0) : 0u;
    const uintptr_t model_addr = model ? reinterpret_cast<uintptr_t>(model + g.e0) : 0u;
    const bool vec_ok = ((out_addr | model_addr) & 15u) == 0;
#pragma unroll
    for (int i = 0; i < G; ++i) {
        const uint32_t e = 4u * (t + (uint32_t)i * T);
        double avg[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) avg[b] = acc[i][b] * inv_u;
        if (vec_ok && e + 3 < g.n) {
            if (out)
                *reinterpret_cast<float4 *>(out + g.e0 + e) =
                    make_float4((float)avg[0], (float)avg[1], (float)avg[2], (float)avg[3]);
            if (model) {
                float4 w = *reinterpret_cast<const float4 *>(model + g.e0 + e);
                w.x = (float)((double)w.x - eta64 * avg[0]);
                w.y = (float)((double)w.y - eta64 * avg[1]);
                w.z = (float)((double)w.z - eta64 * avg[2]);
                w.w = (float)((double)w.w - eta64 * avg[3]);
                *reinterpret_cast<float4 *>(model + g.e0 + e) = w;
            }
        } else {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                if (e + b >= g.n) continue;
                if (out) out[g.e0 + e + b] = (float)avg[b];
                if (model) model[g.e0 + e + b] = (float)((double)model[g.e0 + e + b] - eta64 * avg[b]);
            }
        }
    }
}


// One workgroup per chunk.  The chunk's 4096 sums live in LDS as fp64; W wavefronts decode W users at a time,
// lane j of each taking sub-chunk j, and every decoded symbol's value is added to its element's sum with an
// LDS atomic.  The addends are representatives, so the fp64 sums are exact and their order does not matter as
// long as (2^exp - 2) + mant + 1 + (spread of the users' biases) + log2 U <= 53 (23 - mant more with a gain);
// beyond that the last bit may depend on the order.  The wavefronts meet only twice: after the sums are
// cleared and before they are written out.
template <int W, bool kPerUser>
__global__ __launch_bounds__(64 * W) void k_aggregate(Layout lay, const uint32_t *__restrict__ words,
                                                      uint64_t words_stride,
                                                      const uint64_t *__restrict__ chunk_offset,
                                                      const uint16_t *__restrict__ sub_bits,
                                                      const BookDev *__restrict__ books, float *__restrict__ out,
                                                      float *__restrict__ model, float eta,
                                                      uint64_t *__restrict__ status)
{
    extern __shared__ uint64_t smem64[];
    double *s_acc = reinterpret_cast<double *>(smem64);                    // [64][kAccStride]
    constexpr int T = 64 * W;
    const uint32_t t = threadIdx.x, wave = t >> 6, lane = t & 63u;
    const uint64_t c = blockIdx.x;
    const ChunkGeom g = chunk_geom(lay, c);

    for (uint32_t i = t; i < (uint32_t)kAccWords; i += T) s_acc[i] = 0.0;
    if constexpr (kPerUser) {
        // every user its own code: per-wavefront decode tables and a per-user table of values
        DecLds *s_tab = reinterpret_cast<DecLds *>(s_acc + kAccWords);         // [W]
        uint32_t *s_mag = reinterpret_cast<uint32_t *>(s_tab + W);             // [W][kMagEntries] fp32 patterns
        uint32_t *s_pay = s_mag + W * kMagEntries;                             // [W][kPayloadAlloc]
        const uint32_t sign_shift = (uint32_t)(lay.E + lay.M);
        const uint32_t mag_mask = (1u << sign_shift) - 1u;
        const uint32_t sign_up = 31u - sign_shift;
        __syncthreads();
        // wavefront `wave` takes users wave, wave + W, ...; everything it touches besides the sums is its own
        uint32_t *my_mag = s_mag + wave * kMagEntries;
        uint32_t *my_pay = s_pay + wave * kPayloadAlloc;
        const DecLds *my_tab = s_tab + wave;
        for (uint32_t u = wave; u < lay.U; u += W) {
            const ChunkIndex ix = read_index(lay, c, u, words, words_stride, chunk_offset, sub_bits);
            load_dec_tables(s_tab + wave, books[u * lay.books_per_user + (uint32_t)g.book], lane, 64);
            const int bias = lay.bias[(uint64_t)u * lay.nseg + g.seg];
            const float inv_gain = lay.gain[2 * ((uint64_t)u * lay.nseg + g.seg) + 1];   // 1 unless the plan carries a scale
            for (uint32_t k = lane; k <= mag_mask; k += 64)
                my_mag[k] = __float_as_uint(__fmul_rn(__uint_as_float(symbol_value_bits(k, lay.E, lay.M, bias)), inv_gain));
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            decode_user_chunk(g, ix, my_tab, my_pay, AccSink{s_acc + lane * kAccStride, my_mag, mag_mask, sign_up}, status);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();   // the next user's tables and words overwrite these
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    } else {
        // one code for all users: one table of lengths and values (at bias 0) for the workgroup
        LongLds *s_long = reinterpret_cast<LongLds *>(s_acc + kAccWords);
        uint32_t *s_val = reinterpret_cast<uint32_t *>(s_long + 1);            // [kValEntries]
        uint32_t *s_pay = s_val + kValEntries;                                 // [W][kPayloadAlloc]
        load_value_tables(s_long, s_val, books[(uint32_t)g.book], lay.E, lay.M, t, T);
        __syncthreads();
        uint32_t *my_pay = s_pay + wave * kPayloadAlloc;
        const int first_elem = (int)lane * kSub;
        const int cnt = (int)g.n - first_elem < 0 ? 0 : ((int)g.n - first_elem > kSub ? kSub : (int)g.n - first_elem);
        for (uint32_t u = wave; u < lay.U; u += W) {
            const ChunkIndex ix = read_index(lay, c, u, words, words_stride, chunk_offset, sub_bits);
            const int bias = lay.bias[(uint64_t)u * lay.nseg + g.seg];
            const float inv_gain = lay.gain[2 * ((uint64_t)u * lay.nseg + g.seg) + 1];   // 1 unless the plan carries a scale
            const uint32_t p0 = wave_exclusive_scan_u32(ix.sb);
            uint32_t used = 0;
            if (ix.in_lds) {
                uint32_t tmp[kPayloadPerLane];
                payload_request(ix, tmp);
#pragma unroll
                for (int k = 0; k < kPayloadPerLane; ++k) {
                    const uint32_t i = lane + 64u * k;
                    if (i < ix.nw) my_pay[i] = tmp[k];
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                if (cnt > 0)
                    used = decode_subchunk_acc(LdsWords{my_pay}, p0, cnt, s_long, s_val, lay.E, lay.M, -bias, inv_gain,
                                               s_acc + lane * kAccStride);
            } else if (cnt > 0) {
                used = decode_subchunk_acc(GlobalWords{ix.w, ix.nw}, p0, cnt, s_long, s_val, lay.E, lay.M, -bias, inv_gain,
                                           s_acc + lane * kAccStride);
            }
            if (used != ix.sb || !ix.ok)
                atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CORRUPT), 1ull);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();   // the next user's words overwrite these
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
    __syncthreads();

    // average, and with `model` the PS update w - eta * average (eq. (aggregate hat), Algorithm 1
    // line 14): products and difference in fp64, one rounding
    const double inv_u = 1.0 / (double)lay.U;
    const double eta64 = (double)eta;
    const uintptr_t out_addr = out ? reinterpret_cast<uintptr_t>(out + g.e0) : 0u;
    const uintptr_t model_addr = model ? reinterpret_cast<uintptr_t>(model + g.e0) : 0u;
    const bool vec_ok = ((out_addr | model_addr) & 15u) == 0;
    constexpr int G = (kChunk / 4) / T;  // 4-element groups per thread
#pragma unroll
    for (int i = 0; i < G; ++i) {
        const uint32_t e = 4u * (t + (uint32_t)i * T);                     // elements e .. e + 3: one lane's row
        const double *a = s_acc + (e >> 6) * kAccStride + (e & 63u);
        double avg[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) avg[b] = a[b] * inv_u;
        if (vec_ok && e + 3 < g.n) {
            if (out)
                *reinterpret_cast<float4 *>(out + g.e0 + e) =
                    make_float4((float)avg[0], (float)avg[1], (float)avg[2], (float)avg[3]);
            if (model) {
                float4 w = *reinterpret_cast<const float4 *>(model + g.e0 + e);
                w.x = (float)((double)w.x - eta64 * avg[0]);
                w.y = (float)((double)w.y - eta64 * avg[1]);
                w.z = (float)((double)w.z - eta64 * avg[2]);
                w.w = (float)((double)w.w - eta64 * avg[3]);
                *reinterpret_cast<float4 *>(model + g.e0 + e) = w;
            }
        } else {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                if (e + b >= g.n) continue;
                if (out) out[g.e0 + e + b] = (float)avg[b];
                if (model) model[g.e0 + e + b] = (float)((double)model[g.e0 + e + b] - eta64 * avg[b]);
            }
        }
    }
}

hipError_t launch_decode(const Layout &lay, const co3_decode_args &a, const BookDev *books, hipStream_t s)
{
    if (lay.U == 0 || lay.nchunks == 0) return hipSuccess;
    const uint64_t sym_stride = symbol_row_stride(lay.d);
    const size_t lds = (size_t)(lay.per_user_books ? kDecWaves : 1) * sizeof(DecLds) +
                       (size_t)kDecWaves * (kStageWords + kPayloadAlloc) * 4;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_decode),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    ProfScope prof(K_DECODE, s);
    hipLaunchKernelGGL(k_decode, dim3((uint32_t)lay.nchunks, (lay.U + kDecWaves - 1) / kDecWaves), dim3(64 * kDecWaves),
                       lds, s, lay, a.words, a.words_stride, a.chunk_offset, a.sub_bits, books, a.symbols, sym_stride,
                       a.q, a.q_stride, a.status);
    return hipGetLastError();
}

template <int W, bool kPerUser>
static hipError_t launch_aggregate_wp(const Layout &lay, const co3_aggregate_args &a, const BookDev *books,
                                      hipStream_t s)
{
    const size_t lds = kPerUser ? (size_t)kAccWords * sizeof(double) + (size_t)W * sizeof(DecLds) +
                                      (size_t)W * (kMagEntries + kPayloadAlloc) * 4
                                : (size_t)kAccWords * sizeof(double) + sizeof(LongLds) +
                                      ((size_t)kValEntries + (size_t)W * kPayloadAlloc) * 4;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_aggregate<W, kPerUser>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    ProfScope prof(K_AGGREGATE, s);
    hipLaunchKernelGGL((k_aggregate<W, kPerUser>), dim3((uint32_t)lay.nchunks), dim3(64 * W), lds, s, lay, a.words,
                       a.words_stride, a.chunk_offset, a.sub_bits, books, a.out, a.model, a.eta, a.status);
    return hipGetLastError();
}

template <int W>
static hipError_t launch_aggregate_w(const Layout &lay, const co3_aggregate_args &a, const BookDev *books,
                                     hipStream_t s)
{
    return lay.per_user_books ? launch_aggregate_wp<W, true>(lay, a, books, s)
                              : launch_aggregate_wp<W, false>(lay, a, books, s);
}

template <int W>
static hipError_t launch_aggregate_staged(const Layout &lay, const co3_aggregate_args &a, const BookDev *books,
                                          hipStream_t s)
{
    const size_t lds = (size_t)(lay.per_user_books ? W : 1) * sizeof(DecLds) +
                       (size_t)W * (kMagEntries + kStageWords + kPayloadAlloc) * 4;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k_aggregate_staged<W>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    ProfScope prof(K_AGGREGATE, s);
    hipLaunchKernelGGL(k_aggregate_staged<W>, dim3((uint32_t)lay.nchunks), dim3(64 * W), lds, s, lay, a.words,
                       a.words_stride, a.chunk_offset, a.sub_bits, books, a.out, a.model, a.eta, a.status);
    return hipGetLastError();
}

hipError_t launch_aggregate(const Layout &lay, const co3_aggregate_args &a, const BookDev *books, hipStream_t s)
{
    if (lay.U == 0 || lay.nchunks == 0) return hipSuccess;
    if (lay.U >= 5) return launch_aggregate_w<8>(lay, a, books, s);
    if (lay.U >= 3) return launch_aggregate_staged<4>(lay, a, books, s);
    if (lay.U == 2) return launch_aggregate_staged<2>(lay, a, books, s);
    return launch_aggregate_staged<1>(lay, a, books, s);
}

}  // namespace co3
