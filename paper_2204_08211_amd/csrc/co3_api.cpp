// Host side of the C ABI declared in include/co3.h: argument checks, plans, code-table sets and
// the launch sequences.  No codec arithmetic happens here except the host Huffman builder that
// co3_build_codebook exposes.
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "co3_internal.h"
#include "quantize_math.h"

using namespace co3;

// Workspace of co3_encode_static: one array per GPU, part of the library's code object, so that the
// call needs no allocation.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the device address it yields (one per device) is what kernels and copies get.
static __device__ __align__(256) unsigned char scratch[CO3_STATIC_SCRATCH_BYTES];

namespace {

struct DeviceGuard {
    int prev = 0;
    bool switched = false;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) == hipSuccess && prev != dev) switched = hipSetDevice(dev) == hipSuccess;
    }
    ~DeviceGuard()
    {
        if (switched) (void)hipSetDevice(prev);
    }
};

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, which must be `dev`; resolved once per device.
int scratch_address(int dev, void **out)
{
    if (dev < 0 || dev >= kMaxDevices) return CO3_ERR_ARG;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return CO3_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return CO3_OK;
}

int check_bias_table(const co3_format &f, const int32_t *bias, size_t n)
{
    for (size_t i = 0; i < n; ++i)
        if (!format_supported(f.exp_bits, f.mant_bits, bias[i])) return CO3_ERR_FORMAT;
    return CO3_OK;
}

}  // namespace

namespace co3 {

static inline size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t three_step_workspace_min(const Layout &l)
{
    return up256((size_t)kHistGlobalRep * l.nbooks * l.A * sizeof(uint64_t)) +
           up256((size_t)l.U * l.nchunks * sizeof(uint32_t)) + 512;
}

size_t three_step_workspace_full(const Layout &l)
{
    size_t n = three_step_workspace_min(l);
    if (l.nseg == 1) n += up256((size_t)l.U * l.nchunks * l.A * sizeof(uint16_t));
    return n;
}

EncodeWs three_step_workspace(const Layout &l, void *workspace, size_t bytes)
{
    EncodeWs ws;
    uintptr_t p = (reinterpret_cast<uintptr_t>(workspace) + 255u) & ~(uintptr_t)255u;
    ws.hist_rep = reinterpret_cast<uint64_t *>(p);
    p += up256((size_t)kHistGlobalRep * l.nbooks * l.A * sizeof(uint64_t));
    ws.chunk_bits = reinterpret_cast<uint32_t *>(p);
    p += up256((size_t)l.U * l.nchunks * sizeof(uint32_t));
    ws.chunk_hist = (l.nseg == 1 && bytes >= three_step_workspace_full(l)) ? reinterpret_cast<uint16_t *>(p) : nullptr;
    return ws;
}

}  // namespace co3

extern "C" {

const char *co3_status_string(int status)
{
    switch (status) {
        case CO3_OK: return "CO3_OK";
        case CO3_ERR_ARG: return "CO3_ERR_ARG";
        case CO3_ERR_FORMAT: return "CO3_ERR_FORMAT";
        case CO3_ERR_CAPACITY: return "CO3_ERR_CAPACITY";
        case CO3_ERR_CODELEN: return "CO3_ERR_CODELEN";
        case CO3_ERR_CORRUPT: return "CO3_ERR_CORRUPT";
        case CO3_ERR_HIP: return "CO3_ERR_HIP";
        default: return "CO3_ERR_UNKNOWN";
    }
}

int co3_plan_create(co3_format format, uint32_t U, uint64_t d, uint32_t nseg, const co3_segment *segments,
                    const int32_t *bias, int32_t per_user_books, co3_plan **out)
{
    if (!out || !bias || U == 0 || U > 65535u) return CO3_ERR_ARG;  // users are the second grid dimension
    *out = nullptr;
    if (format.exp_bits < 2 || format.mant_bits < 0 || 1 + format.exp_bits + format.mant_bits > 12)
        return CO3_ERR_FORMAT;
    co3_segment whole = {0, d, 0, 0};
    if (!segments) { segments = &whole; nseg = 1; }
    if (nseg == 0 || nseg > (1u << 20)) return CO3_ERR_ARG;
    std::vector<SegDev> segs(nseg + 1);
    uint64_t off = 0, chunks = 0;
    int32_t max_book = 0;
    for (uint32_t k = 0; k < nseg; ++k) {
        if (segments[k].offset != off || segments[k].codebook < 0 || segments[k].codebook >= (1 << 16))
            return CO3_ERR_ARG;
        if (off + segments[k].length < off) return CO3_ERR_ARG;
        segs[k] = {off, segments[k].length, chunks, segments[k].codebook, 0};
        off += segments[k].length;
        chunks += (segments[k].length + kChunk - 1) / kChunk;
        if (segments[k].codebook > max_book) max_book = segments[k].codebook;
    }
    if (off != d) return CO3_ERR_ARG;
    if (chunks >= (1ull << 31)) return CO3_ERR_ARG;  // one workgroup per chunk in grid.x
    segs[nseg] = {d, 0, chunks, 0, 0};
    int rc = check_bias_table(format, bias, (size_t)U * nseg);
    if (rc != CO3_OK) return rc;

    co3_plan *p = new (std::nothrow) co3_plan;
    if (!p) return CO3_ERR_ARG;
    if (hipGetDevice(&p->device) != hipSuccess) { delete p; return CO3_ERR_HIP; }
    {
        // set-up is the place to resolve the static workspace's address on this device, so that
        // co3_encode_static itself only looks it up
        // (a failure here is reported by co3_encode_static, the only call that needs the address)
        void *unused = nullptr;
        (void)scratch_address(p->device, &unused);
    }
    const std::vector<float> ones((size_t)U * nseg * 2, 1.0f);
    if (hipMalloc(&p->d_segs, sizeof(SegDev) * (nseg + 1)) != hipSuccess ||
        hipMalloc(&p->d_bias, sizeof(int32_t) * (size_t)U * nseg) != hipSuccess ||
        hipMalloc(&p->d_gain, sizeof(float) * ones.size()) != hipSuccess ||
        hipMemcpy(p->d_segs, segs.data(), sizeof(SegDev) * (nseg + 1), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(p->d_bias, bias, sizeof(int32_t) * (size_t)U * nseg, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(p->d_gain, ones.data(), sizeof(float) * ones.size(), hipMemcpyHostToDevice) != hipSuccess) {
        co3_plan_destroy(p);
        return CO3_ERR_HIP;
    }
    Layout &l = p->lay;
    l.U = U; l.nseg = nseg; l.d = d; l.nchunks = chunks;
    l.E = format.exp_bits; l.M = format.mant_bits;
    l.A = 1u << (1 + format.exp_bits + format.mant_bits);
    l.wide = l.A > (uint32_t)kMaxA ? 1u : 0u;
    l.vec_aligned = 1u;
    l.tile_aligned = 1u;
    for (uint32_t k = 0; k < nseg; ++k) {
        if (segs[k].length && (segs[k].offset & 3u)) l.vec_aligned = 0u;
        if (segs[k].length && (segs[k].offset & 2047u)) l.tile_aligned = 0u;
    }
    l.books_per_user = (uint32_t)max_book + 1;
    l.per_user_books = per_user_books ? 1u : 0u;
    l.nbooks = l.books_per_user * (per_user_books ? U : 1u);
    l.segs = p->d_segs;
    l.bias = p->d_bias;
    l.gain = p->d_gain;
    *out = p;
    return CO3_OK;
}

int co3_plan_set_bias(co3_plan *plan, const int32_t *bias, void *stream)
{
    if (!plan || !bias) return CO3_ERR_ARG;
    const size_t n = (size_t)plan->lay.U * plan->lay.nseg;
    co3_format f = {plan->lay.E, plan->lay.M};
    int rc = check_bias_table(f, bias, n);
    if (rc != CO3_OK) return rc;
    DeviceGuard guard(plan->device);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(plan->d_bias, bias, sizeof(int32_t) * n, hipMemcpyHostToDevice, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return CO3_ERR_HIP;
    return CO3_OK;
}

int co3_plan_set_gain(co3_plan *plan, const float *gain, const float *inv_gain, void *stream)
{
    if (!plan || (gain == nullptr) != (inv_gain == nullptr)) return CO3_ERR_ARG;
    const size_t n = (size_t)plan->lay.U * plan->lay.nseg;
    std::vector<float> pairs(2 * n, 1.0f);
    bool any = false;
    for (size_t i = 0; gain && i < n; ++i) {
        // positive normal fp32 numbers only
        if (!(gain[i] >= 1.17549435e-38f && gain[i] <= 3.4e38f) || !(inv_gain[i] >= 1.17549435e-38f && inv_gain[i] <= 3.4e38f))
            return CO3_ERR_ARG;
        pairs[2 * i] = gain[i];
        pairs[2 * i + 1] = inv_gain[i];
        any = any || gain[i] != 1.0f || inv_gain[i] != 1.0f;
    }
    DeviceGuard guard(plan->device);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(plan->d_gain, pairs.data(), sizeof(float) * pairs.size(), hipMemcpyHostToDevice, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return CO3_ERR_HIP;
    plan->has_gain = any;
    return CO3_OK;
}

void co3_plan_destroy(co3_plan *plan)
{
    if (!plan) return;
    DeviceGuard guard(plan->device);
    if (plan->d_segs) (void)hipFree(plan->d_segs);
    if (plan->d_bias) (void)hipFree(plan->d_bias);
    if (plan->d_gain) (void)hipFree(plan->d_gain);
    delete plan;
}

uint64_t co3_plan_num_chunks(const co3_plan *plan) { return plan ? plan->lay.nchunks : 0; }
uint32_t co3_plan_num_books(const co3_plan *plan) { return plan ? plan->lay.nbooks : 0; }
uint32_t co3_plan_alphabet(const co3_plan *plan) { return plan ? plan->lay.A : 0; }

size_t co3_plan_symbols_bytes(const co3_plan *plan)
{
    if (!plan) return 0;
    const uint64_t stride = symbol_row_stride(plan->lay.d);
    return (size_t)(stride * plan->lay.U + 16) * (plan->lay.wide ? 2u : 1u);   // 16-bit symbols above 8 bits
}

size_t co3_plan_workspace_bytes(const co3_plan *plan)
{
    if (!plan) return 0;
    const Layout &l = plan->lay;
    if (l.wide) return wide_workspace_bytes(l);
    const size_t three_step = three_step_workspace_full(l);
    const size_t single_sweep = fused_workspace_bytes(l);
    return three_step > single_sweep ? three_step : single_sweep;
}

// What co3_encode_static needs of its static array: the encoders' smallest workspace.
static size_t workspace_bytes_min(const Layout &l)
{
    if (l.wide) return wide_workspace_bytes(l);
    const size_t three_step = three_step_workspace_min(l);
    const size_t single_sweep = fused_workspace_bytes(l);
    return three_step > single_sweep ? three_step : single_sweep;
}

uint64_t co3_plan_stream_words(const co3_plan *plan, uint32_t max_code_len)
{
    if (!plan) return 0;
    if (max_code_len > CO3_MAX_CODE_LEN) max_code_len = CO3_MAX_CODE_LEN;
    // every chunk rounds up to a whole word
    return (plan->lay.d * max_code_len + 31) / 32 + plan->lay.nchunks + 1;
}

int co3_build_codebook(co3_format format, uint32_t nbooks, const uint64_t *weights, co3_codebook **out)
{
    if (!out || nbooks == 0) return CO3_ERR_ARG;
    *out = nullptr;
    if (format.exp_bits < 2 || format.mant_bits < 0 || 1 + format.exp_bits + format.mant_bits > 12)
        return CO3_ERR_FORMAT;
    const uint32_t A = 1u << (1 + format.exp_bits + format.mant_bits);
    const bool wide = A > (uint32_t)kMaxA;
    std::vector<BookDev> host(wide ? 0 : nbooks);
    std::vector<BookWide> host_wide(wide ? nbooks : 0);
    if (wide) {
        std::memset(host_wide.data(), 0, sizeof(BookWide) * nbooks);
        for (uint32_t b = 0; weights && b < nbooks; ++b) {
            int rc = build_wide_host(weights + (size_t)b * A, A, &host_wide[b]);
            if (rc != CO3_OK) return rc;
        }
    } else {
        std::memset(host.data(), 0, sizeof(BookDev) * nbooks);
        for (auto &b : host)   // a table not built yet has no codes at all
            for (uint32_t s = 0; s < (uint32_t)kMaxA; ++s) b.fast[s] = kFastSlow << 24;
        for (uint32_t b = 0; weights && b < nbooks; ++b) {
            int rc = build_book_host(weights + (size_t)b * A, A, &host[b]);
            if (rc != CO3_OK) return rc;
        }
    }
    co3_codebook *cb = new (std::nothrow) co3_codebook;
    if (!cb) return CO3_ERR_ARG;
    cb->format = format;
    cb->nbooks = nbooks;
    cb->A = A;
    bool ok = hipGetDevice(&cb->device) == hipSuccess;
    if (ok && wide)
        ok = hipMalloc(&cb->d_wide, sizeof(BookWide) * nbooks) == hipSuccess &&
             hipMemcpy(cb->d_wide, host_wide.data(), sizeof(BookWide) * nbooks, hipMemcpyHostToDevice) == hipSuccess;
    else if (ok)
        ok = hipMalloc(&cb->d_books, sizeof(BookDev) * nbooks) == hipSuccess &&
             hipMemcpy(cb->d_books, host.data(), sizeof(BookDev) * nbooks, hipMemcpyHostToDevice) == hipSuccess;
    if (!ok) {
        co3_codebook_destroy(cb);
        return CO3_ERR_HIP;
    }
    *out = cb;
    return CO3_OK;
}

int co3_build_codebook_device(co3_codebook *books, const uint64_t *weights, uint64_t *status, void *stream)
{
    if (!books || !weights || !status) return CO3_ERR_ARG;
    DeviceGuard guard(books->device);
    hipError_t e = books->d_wide
                       ? launch_build_books_wide(books->d_wide, books->nbooks, books->A, weights, status,
                                                 static_cast<hipStream_t>(stream))
                       : launch_build_books(books->d_books, books->nbooks, books->A, weights, status,
                                            static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CO3_OK : CO3_ERR_HIP;
}

int co3_codebook_export(const co3_codebook *books, uint32_t book, uint8_t *len, uint64_t *code, void *stream)
{
    if (!books || book >= books->nbooks || !len || !code) return CO3_ERR_ARG;
    DeviceGuard guard(books->device);
    hipStream_t s = static_cast<hipStream_t>(stream);
    int rc = CO3_OK;
    if (books->d_wide) {
        BookWide *h = new (std::nothrow) BookWide;
        if (!h) return CO3_ERR_ARG;
        if (hipMemcpyAsync(h, books->d_wide + book, sizeof(BookWide), hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess)
            rc = CO3_ERR_HIP;
        else {
            std::memcpy(len, h->len, books->A);
            std::memcpy(code, h->code, sizeof(uint64_t) * books->A);
        }
        delete h;
        return rc;
    }
    BookDev *h = new (std::nothrow) BookDev;
    if (!h) return CO3_ERR_ARG;
    if (hipMemcpyAsync(h, books->d_books + book, sizeof(BookDev), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        rc = CO3_ERR_HIP;
    else {
        std::memcpy(len, h->len, books->A);
        std::memcpy(code, h->code, sizeof(uint64_t) * books->A);
    }
    delete h;
    return rc;
}

uint32_t co3_codebook_num_books(const co3_codebook *books) { return books ? books->nbooks : 0; }

void co3_codebook_destroy(co3_codebook *books)
{
    if (!books) return;
    DeviceGuard guard(books->device);
    if (books->d_books) (void)hipFree(books->d_books);
    if (books->d_wide) (void)hipFree(books->d_wide);
    delete books;
}

static int check_books(const co3_plan *plan, const co3_codebook *books)
{
    if (!books) return CO3_ERR_ARG;
    if (books->nbooks != plan->lay.nbooks || books->A != plan->lay.A) return CO3_ERR_ARG;
    if (books->device != plan->device) return CO3_ERR_ARG;
    return CO3_OK;
}

// The user side with its workspace given explicitly (the caller's, or the static array).
static int encode_with_workspace(const co3_plan *plan, const co3_encode_args *a, void *workspace, size_t workspace_bytes,
                                 void *stream)
{
    const Layout &lay = plan->lay;
    // a vector without elements has no sub-chunks: its (empty) sub_bits array may be NULL
    if (!a->g || !a->m || !a->m_out || !a->words || !a->chunk_offset || (!a->sub_bits && lay.nchunks) || !a->payload_bits ||
        !a->status || !workspace)
        return CO3_ERR_ARG;
    if (a->mode != CO3_BOOK_FIXED && a->mode != CO3_BOOK_EMPIRICAL) return CO3_ERR_ARG;
    if (a->rounding != CO3_ROUND_NEAREST && a->rounding != CO3_ROUND_STOCHASTIC) return CO3_ERR_ARG;
    if (a->rounding == CO3_ROUND_STOCHASTIC && plan->has_gain) return CO3_ERR_ARG;  // defined for the closest representative only
    // symbols and hist come as a pair; without them a fixed code is encoded in a single sweep
    // without a symbol buffer a fixed code is encoded in a single sweep (with or without the symbol counts);
    // everything else needs both buffers
    const bool single_sweep = a->mode == CO3_BOOK_FIXED && !a->symbols;
    if (!single_sweep && (!a->symbols || !a->hist)) return CO3_ERR_ARG;
    if (!aligned16(a->g) || !aligned16(a->m) || !aligned16(a->m_out) || !aligned16(a->symbols) ||
        (a->row_stride & 3u) || a->row_stride < lay.d)
        return CO3_ERR_ARG;
    int rc = check_books(plan, a->books);
    if (rc != CO3_OK) return rc;
    if (workspace_bytes < workspace_bytes_min(lay)) return CO3_ERR_CAPACITY;
    if (!(a->gamma == a->gamma)) return CO3_ERR_ARG;

    co3_encode_args args = *a;
    args.workspace = workspace;
    args.workspace_bytes = workspace_bytes;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (lay.wide) {   // alphabets above 8 bits: a fixed code without a symbol buffer keeps its symbols in the workspace
        return launch_encode_wide(lay, args, a->books->d_wide, workspace, s) == hipSuccess ? CO3_OK : CO3_ERR_HIP;
    }
    if (single_sweep)
        return launch_encode_fused(lay, args, a->books->d_books, s) == hipSuccess ? CO3_OK : CO3_ERR_HIP;
    const EncodeWs ws = three_step_workspace(lay, workspace, workspace_bytes);
    const uint64_t hist_rep_n = (uint64_t)kHistGlobalRep * lay.nbooks * lay.A;

    if (launch_zero_u64(ws.hist_rep, hist_rep_n, s) != hipSuccess) return CO3_ERR_HIP;
    if (launch_quantize(lay, args, ws, s) != hipSuccess) return CO3_ERR_HIP;
    if (a->mode == CO3_BOOK_EMPIRICAL &&
        launch_build_books(a->books->d_books, lay.nbooks, lay.A, a->hist, a->status, s) != hipSuccess)
        return CO3_ERR_HIP;
    if (launch_pack(lay, args, a->books->d_books, ws, s) != hipSuccess) return CO3_ERR_HIP;
    return CO3_OK;
}

int co3_encode(const co3_plan *plan, const co3_encode_args *a, void *stream)
{
    if (!plan || !a) return CO3_ERR_ARG;
    DeviceGuard guard(plan->device);
    return encode_with_workspace(plan, a, a->workspace, a->workspace_bytes, stream);
}

int co3_encode_static(const co3_plan *plan, const co3_encode_args *a, void *stream)
{
    if (!plan || !a) return CO3_ERR_ARG;
    if (workspace_bytes_min(plan->lay) > (size_t)CO3_STATIC_SCRATCH_BYTES) return CO3_ERR_CAPACITY;
    if (profile_enabled()) return CO3_ERR_ARG;   // event timing creates events: not for this entry point
    DeviceGuard guard(plan->device);
    void *ws = nullptr;
    int rc = scratch_address(plan->device, &ws);  // resolved by co3_plan_create; a table look-up here
    if (rc != CO3_OK) return rc;
    return encode_with_workspace(plan, a, ws, (size_t)CO3_STATIC_SCRATCH_BYTES, stream);
}

size_t co3_plan_fit_workspace_bytes(const co3_plan *plan) { return plan ? fit_workspace_bytes(plan->lay) : 0; }

int co3_gennorm_fit(const co3_plan *plan, const float *g, const float *m, uint64_t row_stride, float gamma,
                    co3_gennorm_params *params, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!plan || !g || !m || !params || !workspace) return CO3_ERR_ARG;
    const Layout &lay = plan->lay;
    if (!aligned16(g) || !aligned16(m) || (row_stride & 3u) || row_stride < lay.d) return CO3_ERR_ARG;
    if (!(gamma == gamma)) return CO3_ERR_ARG;
    if (workspace_bytes < fit_workspace_bytes(lay)) return CO3_ERR_CAPACITY;
    DeviceGuard guard(plan->device);
    double *partial = reinterpret_cast<double *>((reinterpret_cast<uintptr_t>(workspace) + 255u) & ~(uintptr_t)255u);
    return launch_fit(lay, g, m, row_stride, gamma, params, partial, static_cast<hipStream_t>(stream)) == hipSuccess
               ? CO3_OK
               : CO3_ERR_HIP;
}

int co3_model_weights_device(const co3_plan *plan, const co3_gennorm_params *params, uint64_t *weights, void *stream)
{
    if (!plan || !params || !weights) return CO3_ERR_ARG;
    DeviceGuard guard(plan->device);
    return launch_model_weights(plan->lay, params, weights, static_cast<hipStream_t>(stream)) == hipSuccess
               ? CO3_OK
               : CO3_ERR_HIP;
}

size_t co3_plan_bias_workspace_bytes(const co3_plan *plan) { return plan ? bias_workspace_bytes(plan->lay) : 0; }

int co3_model_bias_device(const co3_plan *plan, const co3_gennorm_params *params, int32_t *bias, double *error,
                          void *workspace, size_t workspace_bytes, void *stream)
{
    if (!plan || !params || !bias || !workspace) return CO3_ERR_ARG;
    if (workspace_bytes < bias_workspace_bytes(plan->lay)) return CO3_ERR_CAPACITY;
    if (plan->lay.nseg > 65535u || plan->lay.U > 65535u) return CO3_ERR_ARG;  // grid.y, grid.z
    DeviceGuard guard(plan->device);
    double *ws = reinterpret_cast<double *>((reinterpret_cast<uintptr_t>(workspace) + 255u) & ~(uintptr_t)255u);
    return launch_model_bias(plan->lay, params, bias, error, ws, static_cast<hipStream_t>(stream)) == hipSuccess
               ? CO3_OK
               : CO3_ERR_HIP;
}

int co3_plan_set_bias_device(co3_plan *plan, const int32_t *bias, void *stream)
{
    if (!plan || !bias) return CO3_ERR_ARG;
    DeviceGuard guard(plan->device);
    const size_t n = (size_t)plan->lay.U * plan->lay.nseg;
    return hipMemcpyAsync(plan->d_bias, bias, sizeof(int32_t) * n, hipMemcpyDeviceToDevice,
                          static_cast<hipStream_t>(stream)) == hipSuccess
               ? CO3_OK
               : CO3_ERR_HIP;
}

size_t co3_plan_scale_workspace_bytes(const co3_plan *plan) { return plan ? scale_workspace_bytes(plan->lay) : 0; }

int co3_model_scale_device(const co3_plan *plan, const co3_gennorm_params *params, int32_t *bias, float *gain_pairs,
                           double *error, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!plan || !params || !bias || !gain_pairs || !workspace) return CO3_ERR_ARG;
    if (workspace_bytes < scale_workspace_bytes(plan->lay)) return CO3_ERR_CAPACITY;
    if (plan->lay.nseg > 65535u || plan->lay.U > 65535u) return CO3_ERR_ARG;  // grid.y, grid.z
    DeviceGuard guard(plan->device);
    double *ws = reinterpret_cast<double *>((reinterpret_cast<uintptr_t>(workspace) + 255u) & ~(uintptr_t)255u);
    return launch_model_scale(plan->lay, params, bias, gain_pairs, error, ws, static_cast<hipStream_t>(stream)) == hipSuccess
               ? CO3_OK
               : CO3_ERR_HIP;
}

int co3_plan_set_gain_device(co3_plan *plan, const float *gain_pairs, void *stream)
{
    if (!plan || !gain_pairs) return CO3_ERR_ARG;
    DeviceGuard guard(plan->device);
    const size_t n = (size_t)plan->lay.U * plan->lay.nseg;
    if (hipMemcpyAsync(plan->d_gain, gain_pairs, sizeof(float) * 2 * n, hipMemcpyDeviceToDevice,
                       static_cast<hipStream_t>(stream)) != hipSuccess)
        return CO3_ERR_HIP;
    plan->has_gain = true;   // the values are not read back: a scale is taken to be there until the host setter says otherwise
    return CO3_OK;
}

int co3_decode(const co3_plan *plan, const co3_decode_args *a, void *stream)
{
    if (!plan || !a) return CO3_ERR_ARG;
    const Layout &lay = plan->lay;
    if (!a->words || !a->chunk_offset || (!a->sub_bits && lay.nchunks) || !a->status || (!a->symbols && !a->q))
        return CO3_ERR_ARG;
    if (a->q && a->q_stride < lay.d) return CO3_ERR_ARG;
    int rc = check_books(plan, a->books);
    if (rc != CO3_OK) return rc;
    DeviceGuard guard(plan->device);
    const hipError_t e = lay.wide ? launch_decode_wide(lay, *a, a->books->d_wide, static_cast<hipStream_t>(stream))
                                  : launch_decode(lay, *a, a->books->d_books, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CO3_OK : CO3_ERR_HIP;
}

int co3_ps_aggregate(const co3_plan *plan, const co3_aggregate_args *a, void *stream)
{
    if (!plan || !a) return CO3_ERR_ARG;
    const Layout &lay = plan->lay;
    if (!a->words || !a->chunk_offset || (!a->sub_bits && lay.nchunks) || !a->status || (!a->out && !a->model))
        return CO3_ERR_ARG;
    if (a->model && !(a->eta == a->eta)) return CO3_ERR_ARG;
    int rc = check_books(plan, a->books);
    if (rc != CO3_OK) return rc;
    DeviceGuard guard(plan->device);
    const hipError_t e = lay.wide ? launch_aggregate_wide(lay, *a, a->books->d_wide, static_cast<hipStream_t>(stream))
                                  : launch_aggregate(lay, *a, a->books->d_books, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CO3_OK : CO3_ERR_HIP;
}

}  // extern "C"
