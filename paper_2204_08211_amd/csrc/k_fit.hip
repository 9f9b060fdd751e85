// GenNorm parameters of the corrected gradient from the data, and the model code's weights from
// those parameters, without a host round trip (Sec. III eq. (kurtosis): mean, variance and
// kurtosis of GenNorm(mu, alpha, beta); Sec. IV-A (ii): the Huffman code is designed under the
// GenNorm assumption; Sec. VI: the fitted parameters are then held for several epochs).
//
//   k_moments        one read sweep over g and m: per chunk the sums of v, v^2, v^3, v^4 in fp64,
//                    v = fl32(g + fl32(gamma m)) (eq. (f_error_fb)); a wavefront owns a chunk, a
//                    lane adds its elements in index order, the wavefront folds the lanes in a
//                    fixed order: the sums do not depend on scheduling
//   k_fit_params     per (user, layer): folds the chunk sums in a fixed order, central moments,
//                    beta from the kurtosis by bisection, alpha from the variance
//   k_model_weights  per code table: the element-count-weighted mixture of the quantized models
//                    of the (user, layer) pairs the table serves -> integer Huffman weights
//
// The raw-moment route loses about (mu / sigma)^4 ulps of the fourth central moment to
// cancellation; gradient layers have |mu| << sigma.
// HBM traffic of k_moments per element: read g (4) + read m (4).
#include "co3_internal.h"
#include "gennorm_math.h"

namespace co3 {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kMoWaves = 4;                 // wavefronts (chunks) per workgroup
constexpr int kMoThreads = 64 * kMoWaves;
constexpr int kFitThreads = 256;

__device__ inline uint32_t fit_find_chunk_segment(const SegDev *segs, uint32_t nseg, uint64_t chunk)
{
    uint32_t lo = 0, hi = nseg;  // segs[nseg].chunk_start = nchunks > chunk
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (segs[mid].chunk_start <= chunk) lo = mid; else hi = mid;
    }
    return lo;
}

struct Sums4 {
    double s1, s2, s3, s4;
    __device__ inline void add(float vf)
    {
        const double v = (double)vf, v2 = v * v;  // v2 is exact
        s1 += v;
        s2 += v2;
        s3 += v2 * v;
        s4 += v2 * v2;
    }
};

__global__ __launch_bounds__(kMoThreads) void k_moments(Layout lay, const float *__restrict__ g,
                                                        const float *__restrict__ m, uint64_t row_stride,
                                                        float gamma, double *__restrict__ partial)
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint64_t c = (uint64_t)blockIdx.x * kMoWaves + wave;
    const uint32_t u = blockIdx.y;
    if (c >= lay.nchunks) return;  // whole wavefront; no workgroup barriers below
    const uint32_t seg = fit_find_chunk_segment(lay.segs, lay.nseg, c);
    const SegDev sd = lay.segs[seg];
    const uint64_t e0 = sd.offset + (c - sd.chunk_start) * kChunk;
    const uint64_t left = sd.offset + sd.length - e0;
    const uint32_t n = left < (uint64_t)kChunk ? (uint32_t)left : (uint32_t)kChunk;
    const float *gu = g + (uint64_t)u * row_stride + e0;
    const float *mu = m + (uint64_t)u * row_stride + e0;

    // every lane adds its elements in a fixed order: four consecutive ones at a time on the vector
    // path, every 64th element of the chunk otherwise
    Sums4 acc = {0.0, 0.0, 0.0, 0.0};
    if (n == (uint32_t)kChunk && (e0 & 3u) == 0) {
#pragma unroll 4
        for (int r = 0; r < kChunk / 4 / 64; ++r) {
            const uint32_t i = 4u * (lane + 64u * r);
            const f4 gv = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(gu + i));
            const f4 mv = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(mu + i));
#pragma unroll
            for (int j = 0; j < 4; ++j) acc.add(__fadd_rn(gv[j], __fmul_rn(gamma, mv[j])));
        }
    } else {
        for (uint32_t i = lane; i < n; i += 64) acc.add(__fadd_rn(gu[i], __fmul_rn(gamma, mu[i])));
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        acc.s1 += __shfl_xor(acc.s1, o, 64);
        acc.s2 += __shfl_xor(acc.s2, o, 64);
        acc.s3 += __shfl_xor(acc.s3, o, 64);
        acc.s4 += __shfl_xor(acc.s4, o, 64);
    }
    if (lane == 0) {
        double *p = partial + ((uint64_t)u * lay.nchunks + c) * 4;
        p[0] = acc.s1; p[1] = acc.s2; p[2] = acc.s3; p[3] = acc.s4;
    }
}

__global__ __launch_bounds__(kFitThreads) void k_fit_params(Layout lay, const double *__restrict__ partial,
                                                            co3_gennorm_params *__restrict__ params)
{
    __shared__ double s_red[4][kFitThreads];
    const uint32_t seg = blockIdx.x, u = blockIdx.y, t = threadIdx.x;
    const uint64_t cs = lay.segs[seg].chunk_start, ce = lay.segs[seg + 1].chunk_start;
    double a[4] = {0.0, 0.0, 0.0, 0.0};
    for (uint64_t c = cs + t; c < ce; c += kFitThreads) {
        const double *p = partial + ((uint64_t)u * lay.nchunks + c) * 4;
#pragma unroll
        for (int j = 0; j < 4; ++j) a[j] += p[j];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) s_red[j][t] = a[j];
    __syncthreads();
    for (int o = kFitThreads / 2; o > 0; o >>= 1) {
        if (t < (uint32_t)o) {
#pragma unroll
            for (int j = 0; j < 4; ++j) s_red[j][t] += s_red[j][t + o];
        }
        __syncthreads();
    }
    if (t != 0) return;
    co3_gennorm_params out = {0.0, 0.0, 0.0, 0.0};
    const uint64_t n = lay.segs[seg].length;
    if (n > 0) {
        const double dn = (double)n;
        const double S1 = s_red[0][0], S2 = s_red[1][0], S3 = s_red[2][0], S4 = s_red[3][0];
        const double mean = S1 / dn, ms = S2 / dn;
        const double m2 = ms - mean * mean;
        const double m4 = (S4 - 4.0 * mean * S3 + 6.0 * mean * mean * S2) / dn - 3.0 * mean * mean * mean * mean;
        out.mu = mean;
        // a variance below 2^-40 of the mean square is rounding noise of the raw sums: constant layer
        if (m2 > ms * 9.094947017729282e-13) {
            out.kurtosis = m4 / (m2 * m2);
            out.beta = beta_of_kurtosis(out.kurtosis);
            out.alpha = sqrt(m2 / variance_factor(out.beta));
        }
    }
    params[(uint64_t)u * lay.nseg + seg] = out;
}

__global__ __launch_bounds__(kMaxA) void k_model_weights(Layout lay, const co3_gennorm_params *__restrict__ params,
                                                         uint64_t *__restrict__ weights)
{
    const uint32_t b = blockIdx.x;
    const uint32_t u_first = lay.per_user_books ? b / lay.books_per_user : 0u;
    const uint32_t u_last = lay.per_user_books ? u_first : lay.U - 1u;
    const int32_t book = (int32_t)(lay.per_user_books ? b % lay.books_per_user : b);
    for (uint32_t s = threadIdx.x; s < lay.A; s += kMaxA) {   // one symbol per thread up to 8 bits, up to 16 above
        double lo, hi;
        const bool producible = symbol_cell(s, lay.E, lay.M, lay.bias[0], &lo, &hi);  // the same for every bias
        double mass = 0.0, count = 0.0;
        if (producible) {
            for (uint32_t u = u_first; u <= u_last; ++u) {
                for (uint32_t k = 0; k < lay.nseg; ++k) {
                    const SegDev sd = lay.segs[k];
                    if (sd.book != book || sd.length == 0) continue;
                    const co3_gennorm_params p = params[(uint64_t)u * lay.nseg + k];
                    if (!(p.alpha > 0.0) || !(p.beta > 0.0)) continue;
                    symbol_cell(s, lay.E, lay.M, lay.bias[(uint64_t)u * lay.nseg + k], &lo, &hi);
                    // with a real-valued scale the conversion sees y = v * gain: the model's location and scale times gain
                    const double gn = (double)lay.gain[2 * ((uint64_t)u * lay.nseg + k)];
                    mass += (double)sd.length * gennorm_mass(lo, hi, p.mu * gn, p.alpha * gn, p.beta);
                    count += (double)sd.length;
                }
            }
        }
        uint64_t w = 0;
        if (producible) {
            w = 1;
            if (count > 0.0) {
                const double x = floor(mass / count * 1099511627776.0);  // 2^40
                if (x >= 1.0) w = (uint64_t)x;
            }
        }
        weights[(uint64_t)b * lay.A + s] = w;
    }
}

// Exponent bias from the model, eq. (exp bias) with integer b.  The expected squared error of a candidate
// bias is a sum of non-negative shares, one per symbol's cell, so any few shares bound it from below:
//   k_model_bias_bounds  per (user, layer), thread per candidate: the shares of the zero cell and of the two
//                        outermost cells (too coarse a set loses in the first, too narrow a one in the others)
//   k_model_bias_ref     per (user, layer): the candidate with the smallest bound, evaluated in full; no
//                        candidate whose bound exceeds that error can be the minimum or tie with it
//   k_model_bias_errors  workgroup per (candidate bias, layer, user), thread per symbol: every thread
//                        integrates (x - r)^2 f(x) over its symbol's cell, the workgroup folds the
//                        shares in a fixed order -> expected squared error of the candidate; candidates
//                        ruled out by their bound leave at once (a handful of the 226 remain)
//   k_model_bias_pick    per (user, layer): the smallest bias whose error is within kBiasTie of the
//                        minimum (a format with many binades has a plateau of equally good biases;
//                        the smallest has the most headroom).  No model (alpha = 0): the IEEE bias.
constexpr int kBiasSlots = 256;  // error slots per (user, layer); candidates: at most 226
constexpr double kBiasPrune = 1e-6;  // margin of the bound test, far above the rounding of the sums and the tie width

// the workgroup's sum of one value per thread, folded in a fixed order
__device__ inline double bias_fold(double *s_red, uint32_t t, double e)
{
    s_red[t] = e;
    __syncthreads();
    for (int o = kMaxA / 2; o > 0; o >>= 1) {
        if (t < (uint32_t)o) s_red[t] += s_red[t + o];
        __syncthreads();
    }
    const double r = s_red[0];
    __syncthreads();
    return r;
}

__global__ __launch_bounds__(kMaxA) void k_model_bias_bounds(Layout lay, const co3_gennorm_params *__restrict__ params,
                                                             double *__restrict__ bounds)
{
    const uint32_t seg = blockIdx.x, u = blockIdx.y, cand = threadIdx.x;
    const co3_gennorm_params p = params[(uint64_t)u * lay.nseg + seg];
    const int ncand = kBiasMax - bias_min_supported(lay.E) + 1;
    if ((int)cand >= ncand) return;
    double lb = INFINITY;
    if (p.alpha > 0.0 && p.beta > 0.0) {
        const int bias = bias_min_supported(lay.E) + (int)cand;
        const uint32_t top = (((1u << lay.E) - 1u) << lay.M) - 1u;        // largest magnitude code
        lb = sq_error_of_symbol(0u, lay.E, lay.M, bias, p.mu, p.alpha, p.beta) +
             sq_error_of_symbol(top, lay.E, lay.M, bias, p.mu, p.alpha, p.beta) +
             sq_error_of_symbol((1u << (lay.E + lay.M)) | top, lay.E, lay.M, bias, p.mu, p.alpha, p.beta);
    }
    bounds[((uint64_t)u * lay.nseg + seg) * kBiasSlots + cand] = lb;
}

__global__ __launch_bounds__(kMaxA) void k_model_bias_ref(Layout lay, const co3_gennorm_params *__restrict__ params,
                                                          const double *__restrict__ bounds, double *__restrict__ ref)
{
    __shared__ double s_red[kMaxA];
    __shared__ int s_c0;
    const uint32_t seg = blockIdx.x, u = blockIdx.y, t = threadIdx.x;
    const co3_gennorm_params p = params[(uint64_t)u * lay.nseg + seg];
    const bool model = p.alpha > 0.0 && p.beta > 0.0;
    const int ncand = kBiasMax - bias_min_supported(lay.E) + 1;
    if (t == 0) {
        const double *lb = bounds + ((uint64_t)u * lay.nseg + seg) * kBiasSlots;
        int c0 = 0;
        for (int c = 1; c < ncand; ++c) c0 = lb[c] < lb[c0] ? c : c0;
        s_c0 = c0;
    }
    __syncthreads();
    double e = 0.0;   // the shares of symbols t, t + 256, ... in this order (one symbol for alphabets of up to 8 bits)
    if (model)
        for (uint32_t sy = t; sy < lay.A; sy += kMaxA)
            e += sq_error_of_symbol(sy, lay.E, lay.M, bias_min_supported(lay.E) + s_c0, p.mu, p.alpha, p.beta);
    const double total = bias_fold(s_red, t, e);
    if (t == 0) ref[(uint64_t)u * lay.nseg + seg] = model ? total : INFINITY;
}

__global__ __launch_bounds__(kMaxA) void k_model_bias_errors(Layout lay, const co3_gennorm_params *__restrict__ params,
                                                             const double *__restrict__ bounds,
                                                             const double *__restrict__ ref, double *__restrict__ errors)
{
    __shared__ double s_red[kMaxA];
    const uint32_t cand = blockIdx.x, seg = blockIdx.y, u = blockIdx.z, t = threadIdx.x;
    const uint64_t pair = (uint64_t)u * lay.nseg + seg;
    const co3_gennorm_params p = params[pair];
    const bool model = p.alpha > 0.0 && p.beta > 0.0;
    // uniform over the workgroup: a candidate whose lower bound lies above the reference error cannot win or tie
    if (!model || bounds[pair * kBiasSlots + cand] > ref[pair] * (1.0 + kBiasPrune)) {
        if (t == 0) errors[pair * kBiasSlots + cand] = INFINITY;
        return;
    }
    double e = 0.0;
    for (uint32_t sy = t; sy < lay.A; sy += kMaxA)
        e += sq_error_of_symbol(sy, lay.E, lay.M, bias_min_supported(lay.E) + (int)cand, p.mu, p.alpha, p.beta);
    const double total = bias_fold(s_red, t, e);
    if (t == 0) errors[pair * kBiasSlots + cand] = total;
}

__global__ __launch_bounds__(64) void k_model_bias_pick(Layout lay, const double *__restrict__ errors,
                                                        int32_t *__restrict__ bias_out, double *__restrict__ error_out)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;  // (user, layer) pair
    if (i >= (uint64_t)lay.U * lay.nseg) return;
    const double *err = errors + i * kBiasSlots;
    const int b0 = bias_min_supported(lay.E);
    const int ncand = kBiasMax - b0 + 1;
    int best = (1 << (lay.E - 1)) - 1;
    double best_err = 0.0, lowest = INFINITY;
    for (int c = 0; c < ncand; ++c) lowest = err[c] < lowest ? err[c] : lowest;
    if (lowest < INFINITY) {
        const double limit = lowest * (1.0 + kBiasTie);
        for (int c = 0; c < ncand; ++c) {
            if (err[c] <= limit) { best = b0 + c; best_err = err[c]; break; }
        }
    }
    bias_out[i] = best;
    if (error_out) error_out[i] = best_err;
}

// errors and bounds per candidate, reference error per pair
size_t bias_workspace_bytes(const Layout &lay) { return (size_t)lay.U * lay.nseg * (2 * kBiasSlots + 1) * sizeof(double) + 256; }

hipError_t launch_model_bias(const Layout &lay, const co3_gennorm_params *params, int32_t *bias, double *error,
                             double *errors_ws, hipStream_t s)
{
    if (lay.U == 0) return hipSuccess;
    const int ncand = kBiasMax - bias_min_supported(lay.E) + 1;
    ProfScope prof(K_MODEL_BIAS, s);
    const uint64_t pairs = (uint64_t)lay.U * lay.nseg;
    double *bounds = errors_ws + pairs * kBiasSlots, *ref = bounds + pairs * kBiasSlots;
    hipLaunchKernelGGL(k_model_bias_bounds, dim3(lay.nseg, lay.U), dim3(kMaxA), 0, s, lay, params, bounds);
    hipLaunchKernelGGL(k_model_bias_ref, dim3(lay.nseg, lay.U), dim3(kMaxA), 0, s, lay, params, bounds, ref);
    hipLaunchKernelGGL(k_model_bias_errors, dim3((uint32_t)ncand, lay.nseg, lay.U), dim3(kMaxA), 0, s, lay, params,
                       bounds, ref, errors_ws);
    hipLaunchKernelGGL(k_model_bias_pick, dim3((uint32_t)((pairs + 63) / 64)), dim3(64), 0, s, lay, errors_ws, bias,
                       error);
    return hipGetLastError();
}

// eq. (exp bias) with b over the reals, per (user, layer), from the integer optimum found above.  A scale c = 2^t
// on top of an integer bias turns the representative set into {c x}; its error on GenNorm(mu, alpha, beta) is c^2
// times the error of the unscaled set on GenNorm(mu / c, alpha / c, beta), so the sum over the symbols' cells
// serves again.  The logarithm s = t - bias of the whole scale is scanned in steps of 1/16 binade over one and a
// half binades to either side of the integer optimum and refined by a golden-section search between the scan
// points next to the best one; bias = -round(s), t = s + bias in [-1/2, 1/2].  One workgroup per (user, layer),
// thread per symbol, every evaluation folded in the same fixed order: all threads see the same numbers and take
// the same steps.  A real scale is taken only where it lowers the error by more than kBiasTie (relative).
__global__ __launch_bounds__(kMaxA) void k_model_scale(Layout lay, const co3_gennorm_params *__restrict__ params,
                                                       int32_t *bias_io, const double *__restrict__ err_int,
                                                       float *__restrict__ gain_pairs, double *error_out)
{
    __shared__ double s_red[kMaxA];
    const uint32_t seg = blockIdx.x, u = blockIdx.y, t = threadIdx.x;
    const uint64_t pair = (uint64_t)u * lay.nseg + seg;
    const co3_gennorm_params p = params[pair];
    const int b_int = bias_io[pair];
    const double e_int = err_int[pair];
    int b_out = b_int;
    float gn = 1.0f, ig = 1.0f;
    double e_out = e_int;
    __syncthreads();   // every thread has read the integer result before thread 0 replaces it
    if (p.alpha > 0.0 && p.beta > 0.0) {   // the same in every thread
        const int bmin = bias_min_supported(lay.E), bmax = kBiasMax;
        auto split = [&](double sc, int &b, double &tt) {
            b = (int)lround(-sc);
            b = b < bmin ? bmin : (b > bmax ? bmax : b);
            tt = sc + (double)b;
        };
        auto err_at = [&](int b, double tt) {
            const double c = exp2(tt);
            double e = 0.0;
            for (uint32_t sy = t; sy < lay.A; sy += kMaxA)
                e += sq_error_of_symbol(sy, lay.E, lay.M, b, p.mu / c, p.alpha / c, p.beta);
            return c * c * bias_fold(s_red, t, e);
        };
        auto f = [&](double sc) {
            int b;
            double tt;
            split(sc, b, tt);
            return err_at(b, tt);
        };
        const double s0 = -(double)b_int;
        const int kHalf = 24;
        double best_s = s0, best_f = e_int;
        int best_k = 0;
        for (int k = -kHalf; k <= kHalf; ++k) {
            const double sc = s0 + (double)k / 16.0, v = f(sc);
            if (v < best_f) { best_f = v; best_s = sc; best_k = k; }
        }
        if (best_k > -kHalf && best_k < kHalf) {
            const double r = 0.6180339887498949;
            double a = best_s - 1.0 / 16.0, b = best_s + 1.0 / 16.0;
            double x1 = b - r * (b - a), x2 = a + r * (b - a), f1 = f(x1), f2 = f(x2);
            for (int it = 0; it < 60; ++it) {
                if (f1 < f2) { b = x2; x2 = x1; f2 = f1; x1 = b - r * (b - a); f1 = f(x1); }
                else { a = x1; x1 = x2; f1 = f2; x2 = a + r * (b - a); f2 = f(x2); }
            }
            const double xm = 0.5 * (a + b), fm = f(xm);
            if (fm < best_f) { best_f = fm; best_s = xm; }
        }
        if (best_f < e_int * (1.0 - kBiasTie)) {
            int b;
            double tt;
            split(best_s, b, tt);
            ig = (float)exp2(tt);
            gn = 1.0f / ig;
            b_out = b;
            e_out = err_at(b, log2((double)ig));   // of the fp32 pair that is returned
        }
    }
    if (t == 0) {
        bias_io[pair] = b_out;
        gain_pairs[2 * pair] = gn;
        gain_pairs[2 * pair + 1] = ig;
        if (error_out) error_out[pair] = e_out;
    }
}

// the integer search's workspace and its expected errors per pair
size_t scale_workspace_bytes(const Layout &lay) { return bias_workspace_bytes(lay) + (size_t)lay.U * lay.nseg * sizeof(double) + 256; }

hipError_t launch_model_scale(const Layout &lay, const co3_gennorm_params *params, int32_t *bias, float *gain_pairs,
                              double *error, double *ws, hipStream_t s)
{
    if (lay.U == 0 || lay.nseg == 0) return hipSuccess;
    const uint64_t pairs = (uint64_t)lay.U * lay.nseg;
    double *err_int = ws;   // [pairs], then the integer search's own workspace (256-byte aligned again)
    double *ws_int = reinterpret_cast<double *>((reinterpret_cast<uintptr_t>(ws + pairs) + 255u) & ~(uintptr_t)255u);
    hipError_t e = launch_model_bias(lay, params, bias, err_int, ws_int, s);
    if (e != hipSuccess) return e;
    ProfScope prof(K_MODEL_BIAS, s);
    hipLaunchKernelGGL(k_model_scale, dim3(lay.nseg, lay.U), dim3(kMaxA), 0, s, lay, params, bias, err_int, gain_pairs,
                       error);
    return hipGetLastError();
}

size_t fit_workspace_bytes(const Layout &lay) { return (size_t)lay.U * lay.nchunks * 4 * sizeof(double) + 256; }

hipError_t launch_fit(const Layout &lay, const float *g, const float *m, uint64_t row_stride, float gamma,
                      co3_gennorm_params *params, double *partial, hipStream_t s)
{
    if (lay.U == 0) return hipSuccess;
    if (lay.nchunks) {
        ProfScope prof(K_MOMENTS, s);
        const uint32_t gx = (uint32_t)((lay.nchunks + kMoWaves - 1) / kMoWaves);
        hipLaunchKernelGGL(k_moments, dim3(gx, lay.U), dim3(kMoThreads), 0, s, lay, g, m, row_stride, gamma, partial);
    }
    ProfScope prof(K_FIT, s);
    hipLaunchKernelGGL(k_fit_params, dim3(lay.nseg, lay.U), dim3(kFitThreads), 0, s, lay, partial, params);
    return hipGetLastError();
}

hipError_t launch_model_weights(const Layout &lay, const co3_gennorm_params *params, uint64_t *weights,
                                hipStream_t s)
{
    if (lay.nbooks == 0) return hipSuccess;
    ProfScope prof(K_MODEL_WEIGHTS, s);
    hipLaunchKernelGGL(k_model_weights, dim3(lay.nbooks), dim3(kMaxA), 0, s, lay, params, weights);
    return hipGetLastError();
}

}  // namespace co3
