// Internal declarations shared by the host API and the HIP kernels of libco3.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "co3.h"

namespace co3 {

constexpr int kChunk = CO3_CHUNK;
constexpr int kSub = CO3_SUB;
constexpr int kSubsPerChunk = CO3_SUBS_PER_CHUNK;
constexpr int kMaxA = 256;          // alphabets of up to 8 bits: symbols are bytes
constexpr int kWideMaxA = 4096;     // alphabets of 9 to 12 bits: symbols are 16-bit words (k_wide.hip)
constexpr int kWideDecBits = 12;    // prefix width of the wide path's direct decode table
constexpr int kWideDec2Bits = 5;    // its second-level tables are indexed by the next bits
constexpr int kWideDec2Tables = 128;   // number of second-level tables
constexpr int kDecBits = 11;        // prefix width of the direct decode table
constexpr int kDecEntries = 1 << kDecBits;
constexpr int kLongSlots = 64 - kDecBits;  // lengths kDecBits+1 .. 64
constexpr int kDec2Bits = 3;        // second-level tables resolve codes of up to kDecBits + kDec2Bits bits
constexpr int kDec2Tables = 40;     // for the first prefixes that hold only longer codes (they are the largest ones)
// Symbols between two users' rows of a symbol buffer: the row length rounded up to 128 symbols, so that rows
// start on 128-byte lines (of a 256-byte-aligned buffer).
inline uint64_t symbol_row_stride(uint64_t d) { return (d + 127) & ~(uint64_t)127; }

constexpr int kHistGlobalRep = 64;   // copies of the global symbol-count table the workgroups spread over
constexpr int kFastLen = 24;        // longest code held in the 32-bit encode entry
constexpr uint32_t kFastSlow = 0xFFu;  // length field marking "use the 64-bit table"

// One Huffman code table as the kernels read it.
struct BookDev {
    uint64_t code[kMaxA];        // right-aligned codeword of each symbol
    uint64_t first[65];          // first[L]: first canonical code of length L (L = 1..64)
    uint32_t fast[kMaxA];        // (len << 24) | code for len <= 24; len field 0xFF: a longer code, or none
    uint32_t count[65];          // count[L]: symbols with length L
    uint32_t offset[65];         // offset[L]: index of the first length-L symbol in sorted[]
    uint16_t dec[kDecEntries];   // prefix -> (len << 8) | symbol for len <= 11; else 1 + its second-level table, or 0
    uint16_t dec2[kDec2Tables << kDec2Bits];  // [table][next kDec2Bits bits] -> (len << 8) | symbol, 0: longer code;
                                 // directly behind dec[]: the decoders index both as one array
    uint8_t len[kMaxA];          // codeword length, 0 = no code
    uint8_t sorted[kMaxA];       // symbols ordered by (length, symbol)
    uint32_t maxlen;
    uint32_t nactive;
    // Lengths above kDecBits that occur, ascending.  A 64-bit left-aligned window w whose code is
    // longer than kDecBits has the first listed length with w <= long_last[k]; its symbol is
    // sorted[(uint32_t)(w >> (64 - len)) + long_base[k]].
    uint32_t nlong;
    uint32_t long_prefix0;       // first kDecBits-bit prefix under which only longer codes live (kDecEntries: none);
                                 // prefix long_prefix0 + j, j < kDec2Tables, has second-level table j
    uint64_t long_last[kLongSlots];   // left-aligned last code of the length, low bits all ones
    uint32_t long_base[kLongSlots];   // offset[len] - first[len] (mod 2^32)
    uint32_t long_len[kLongSlots];
};

// One Huffman code table of a wide alphabet (9 to 12 symbol bits) as the wide kernels read it.
struct BookWide {
    uint64_t code[kWideMaxA];             // right-aligned codeword of each symbol
    uint64_t first[65];                   // first[L]: first canonical code of length L
    uint32_t count[65];                   // symbols with length L
    uint32_t offset[65];                  // index of the first length-L symbol in sorted[]
    uint16_t dec[1 << kWideDecBits];      // prefix -> (len << 12) | symbol for len <= kWideDecBits, else 0
    // the first kWideDec2Tables prefixes that hold only longer codes (the largest prefixes: canonical codes grow
    // with their length) each have a table over the next kWideDec2Bits bits:
    // ((len - kWideDecBits) << 12) | symbol for len <= kWideDecBits + kWideDec2Bits, else 0
    uint16_t dec2[kWideDec2Tables << kWideDec2Bits];
    uint32_t long_prefix0;                // first prefix that holds only longer codes (1 << kWideDecBits: none)
    uint16_t sorted[kWideMaxA];           // symbols ordered by (length, symbol)
    uint8_t len[kWideMaxA];               // codeword length, 0 = no code
    uint32_t maxlen;
    uint32_t nactive;
};

// One layer of the flat vector as the kernels read it.
struct SegDev {
    uint64_t offset;       // first element
    uint64_t length;
    uint64_t chunk_start;  // index of the segment's first chunk within a user
    int32_t book;          // code table id within a user's (or the shared) set
    int32_t pad;
};

// Constants of Q_fp for one (format, bias), derived on the device from E, M and bias.
struct Layout {
    uint32_t U;
    uint32_t nseg;
    uint64_t d;
    uint64_t nchunks;          // per user
    int32_t E, M;
    uint32_t A;
    uint32_t books_per_user;   // 1 + max segment.codebook
    uint32_t per_user_books;
    uint32_t nbooks;           // tables in a set
    uint32_t wide;             // alphabet above 8 bits: 16-bit symbols, the kernels of k_wide.hip
    uint32_t vec_aligned;      // every layer starts at a multiple of 4 elements (16-byte vectors never straddle a layer start)
    uint32_t tile_aligned;     // every layer starts at a multiple of 2048 elements (a tile of the wide quantizer lies in one chunk)
    const SegDev *segs;        // device [nseg + 1] (last entry: offset = d, chunk_start = nchunks)
    const int32_t *bias;       // device [U][nseg]
    const float *gain;         // device [U][nseg][2]: (gain, inv_gain) of the real-valued scale; (1, 1) when unused
};

}  // namespace co3

struct co3_plan {
    co3::Layout lay;
    co3::SegDev *d_segs = nullptr;
    int32_t *d_bias = nullptr;
    float *d_gain = nullptr;
    bool has_gain = false;     // a gain other than (1, 1) was installed
    int device = 0;
};

struct co3_codebook {
    co3_format format;
    uint32_t nbooks = 0;
    uint32_t A = 0;
    co3::BookDev *d_books = nullptr;    // byte alphabets
    co3::BookWide *d_wide = nullptr;    // wide alphabets (exactly one of the two is set)
    int device = 0;
};

namespace co3 {

// Per-kernel event timing (profile.cpp).  A ProfScope around a launch records two events on
// the stream when profiling is on, and does nothing otherwise.
enum KernelId { K_ZERO = 0, K_QUANTIZE, K_REDUCE_HIST, K_BUILD_BOOKS, K_CHUNK_BITS, K_SCAN, K_PACK, K_DECODE, K_AGGREGATE, K_FUSED, K_MOMENTS, K_FIT, K_MODEL_WEIGHTS, K_MODEL_BIAS, K_COUNT };
bool profile_enabled();
class ProfScope {
public:
    ProfScope(int kid, hipStream_t s);
    ~ProfScope();
private:
    int kid_;
    hipStream_t s_;
    hipEvent_t start_;
};

// Host Huffman builder (host_codebook.cpp): fills one table; returns a co3_status.
int build_book_host(const uint64_t *weights, uint32_t A, BookDev *out);
int build_wide_host(const uint64_t *weights, uint32_t A, BookWide *out);

// Kernel launchers (one per .hip file).  All return a hipError_t from hipGetLastError().
struct EncodeWs {
    uint64_t *hist_rep;     // [kHistGlobalRep][nbooks][A] partial symbol counts
    uint32_t *chunk_bits;   // [U][nchunks] payload bits of every chunk
    uint16_t *chunk_hist;   // [U][nchunks][A] symbol counts of every chunk, or nullptr (single-layer vectors only)
};
// bytes of the three-step encoder's workspace: what it cannot do without, and what it takes when it gets it (the
// per-chunk symbol counts spare it a sweep over the symbols)
size_t three_step_workspace_min(const Layout &lay);
size_t three_step_workspace_full(const Layout &lay);
EncodeWs three_step_workspace(const Layout &lay, void *workspace, size_t bytes);

hipError_t launch_zero_u64(uint64_t *p, uint64_t n, hipStream_t s);
hipError_t launch_reduce_hist(const uint64_t *hist_rep, uint64_t *hist, uint64_t n, hipStream_t s);   // hist[i] = sum of the partial tables
hipError_t launch_quantize(const Layout &lay, const co3_encode_args &a, const EncodeWs &ws, hipStream_t s);
hipError_t launch_build_books(BookDev *books, uint32_t nbooks, uint32_t A, const uint64_t *weights,
                              uint64_t *status, hipStream_t s);
hipError_t launch_pack(const Layout &lay, const co3_encode_args &a, const BookDev *books,
                       const EncodeWs &ws, hipStream_t s);
// exclusive scan of the 32-bit-rounded chunk sizes of every user (k_pack.hip), shared with the wide path
hipError_t launch_scan_chunks(const Layout &lay, const uint32_t *chunk_bits, uint64_t *chunk_offset,
                              uint64_t *payload_bits, hipStream_t s);
// single-sweep encoder for a fixed code (k_fused.hip); its workspace need in bytes
hipError_t launch_encode_fused(const Layout &lay, const co3_encode_args &a, const BookDev *books, hipStream_t s);
size_t fused_workspace_bytes(const Layout &lay);
// GenNorm fit and model weights (k_fit.hip); partial: fit_workspace_bytes() of device memory
size_t fit_workspace_bytes(const Layout &lay);
hipError_t launch_fit(const Layout &lay, const float *g, const float *m, uint64_t row_stride, float gamma,
                      co3_gennorm_params *params, double *partial, hipStream_t s);
hipError_t launch_model_weights(const Layout &lay, const co3_gennorm_params *params, uint64_t *weights,
                                hipStream_t s);
size_t bias_workspace_bytes(const Layout &lay);
hipError_t launch_model_bias(const Layout &lay, const co3_gennorm_params *params, int32_t *bias, double *error,
                             double *errors_ws, hipStream_t s);
size_t scale_workspace_bytes(const Layout &lay);
hipError_t launch_model_scale(const Layout &lay, const co3_gennorm_params *params, int32_t *bias, float *gain_pairs,
                              double *error, double *workspace, hipStream_t s);
hipError_t launch_decode(const Layout &lay, const co3_decode_args &a, const BookDev *books, hipStream_t s);
hipError_t launch_aggregate(const Layout &lay, const co3_aggregate_args &a, const BookDev *books,
                            hipStream_t s);
// wide alphabets (k_wide.hip): the same steps with 16-bit symbols and tables in device memory
size_t wide_workspace_bytes(const Layout &lay);
hipError_t launch_encode_wide(const Layout &lay, const co3_encode_args &a, BookWide *books, void *workspace,
                              hipStream_t s);
hipError_t launch_build_books_wide(BookWide *books, uint32_t nbooks, uint32_t A, const uint64_t *weights,
                                   uint64_t *status, hipStream_t s);
hipError_t launch_decode_wide(const Layout &lay, const co3_decode_args &a, const BookWide *books, hipStream_t s);
hipError_t launch_aggregate_wide(const Layout &lay, const co3_aggregate_args &a, const BookWide *books,
                                 hipStream_t s);

}  // namespace co3
