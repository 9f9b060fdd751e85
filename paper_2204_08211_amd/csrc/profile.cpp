// Optional per-kernel timing with HIP events recorded on the caller's stream around every
// kernel the library launches (co3_profile_begin / co3_profile_end in include/co3.h).
#include <atomic>
#include <mutex>
#include <vector>

#include "co3_internal.h"

namespace co3 {

static const char *kKernelNames[K_COUNT] = {"k_zero_u64", "k_quantize", "k_reduce_hist", "k_build_books", "k_chunk_bits",
                                            "k_scan_chunks", "k_pack", "k_decode", "k_aggregate", "k_encode_fused", "k_moments", "k_fit_params",
                                            "k_model_weights", "k_model_bias"};

struct ProfRecord { int kid; hipEvent_t a, b; };
static std::mutex g_mu;
static std::atomic<bool> g_on{false};
static std::vector<ProfRecord> g_recs;

bool profile_enabled() { return g_on; }

ProfScope::ProfScope(int kid, hipStream_t s) : kid_(kid), s_(s), start_(nullptr)
{
    if (!g_on) return;
    if (hipEventCreate(&start_) != hipSuccess) { start_ = nullptr; return; }
    (void)hipEventRecord(start_, s_);
}

ProfScope::~ProfScope()
{
    if (!start_) return;
    hipEvent_t stop;
    if (hipEventCreate(&stop) != hipSuccess) { (void)hipEventDestroy(start_); return; }
    (void)hipEventRecord(stop, s_);
    std::lock_guard<std::mutex> lk(g_mu);
    g_recs.push_back({kid_, start_, stop});
}

}  // namespace co3

using namespace co3;

extern "C" {

int co3_profile_begin(void)
{
    std::lock_guard<std::mutex> lk(g_mu);
    for (auto &r : g_recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    g_recs.clear();
    g_on = true;
    return CO3_OK;
}

int co3_profile_end(co3_kernel_time *out, uint32_t capacity, uint32_t *count)
{
    std::lock_guard<std::mutex> lk(g_mu);
    g_on = false;
    if (hipDeviceSynchronize() != hipSuccess) return CO3_ERR_HIP;
    double ms[K_COUNT] = {0};
    uint64_t n[K_COUNT] = {0};
    for (auto &r : g_recs) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, r.a, r.b) == hipSuccess) { ms[r.kid] += t; n[r.kid]++; }
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    g_recs.clear();
    uint32_t k = 0;
    for (int i = 0; i < K_COUNT && out && k < capacity; ++i) {
        if (!n[i]) continue;
        snprintf(out[k].name, sizeof(out[k].name), "%s", kKernelNames[i]);
        out[k].total_ms = ms[i];
        out[k].launches = n[i];
        ++k;
    }
    if (count) *count = k;
    return CO3_OK;
}

}  // extern "C"
