// Error correction, fp conversion, memory update and symbol histogram in one sweep
// (Algorithm 1 lines 8 and 10; Sec. IV-A (i) and (iii); Sec. V-B for the representative set).
//
// Per element:  v = fl32(g + fl32(gamma * m));  q = Q_fp(v);  m' = fl32(v - q);  sym = code of q.
// HBM traffic per element: read g (4) + read m (4) + write m' (4) + write sym (1) = 13 bytes.
//
// One workgroup of 512 threads per tile of 4096 elements, in memory order, so the tiles in
// flight at any moment form a compact window of addresses (measured: a grid-stride loop over
// the same tiles loses a tenth of the bandwidth).  Streaming data is loaded and stored with
// the nontemporal hint.  Symbol counts go to lane-replicated LDS bins (the peaked symbol
// distribution would otherwise serialise the atomics), are summed per workgroup and added to
// one of kHistGlobalRep copies of the global table, so that no address sees every workgroup;
// k_reduce_hist folds the copies.
#include "co3_internal.h"
#include "quantize_math.h"

namespace co3 {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kQThreads = 512;
constexpr int kQTile = kQThreads * 8;   // two 16-byte vectors of g and of m per thread
constexpr int kHistRep = 32;            // lane-replicated copies of every LDS bin (one per bank)

__device__ inline uint32_t find_segment(const SegDev *segs, uint32_t nseg, uint64_t elem)
{
    // last segment whose offset is <= elem (empty segments share an offset: take the last)
    uint32_t lo = 0, hi = nseg;  // segs[nseg].offset = d > elem
    while (hi - lo > 1) {
        uint32_t mid = (lo + hi) >> 1;
        if (segs[mid].offset <= elem) lo = mid; else hi = mid;
    }
    return lo;
}

// kSR: the stochastic conversion (dither from Philox words of (element, user, seed)) instead of
// the closest representative.
template <bool kSR>
__global__ __launch_bounds__(kQThreads) void k_quantize(
    Layout lay, const float *__restrict__ g, const float *m, float *m_out,
    uint8_t *__restrict__ sym, uint64_t sym_stride, uint64_t row_stride, float gamma, uint64_t seed,
    uint64_t *__restrict__ hist_rep, uint16_t *__restrict__ chunk_hist, uint64_t *__restrict__ status)
{
    extern __shared__ uint32_t h_lds[];  // [A][kHistRep]
    const uint32_t u = blockIdx.y;
    const uint64_t d = lay.d;
    const uint64_t base = (uint64_t)blockIdx.x * kQTile;
    const float *gu = g + (uint64_t)u * row_stride;
    const float *mu = m + (uint64_t)u * row_stride;
    float *mo = m_out + (uint64_t)u * row_stride;
    uint8_t *su = sym + (uint64_t)u * sym_stride;
    const bool full = base + kQTile <= d;

    // request the tile before anything else
    f4 gv[2], mv[2];
    if (full) {
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const uint64_t i = base + (uint64_t)k * (kQThreads * 4) + threadIdx.x * 4;
            gv[k] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(gu + i));
            mv[k] = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(mu + i));
        }
    }
    for (uint32_t i = threadIdx.x; i < lay.A * kHistRep; i += kQThreads) h_lds[i] = 0;

    const uint32_t book_base = lay.per_user_books ? u * lay.books_per_user : 0;
    uint64_t *hist = hist_rep + (uint64_t)(blockIdx.x % kHistGlobalRep) * lay.nbooks * lay.A;
    const uint32_t lane_rep = threadIdx.x & (kHistRep - 1);
    const uint32_t sign_shift = lay.E + lay.M;
    const uint32_t seg = find_segment(lay.segs, lay.nseg, base);
    const uint64_t seg_end = lay.segs[seg + 1].offset;
    uint32_t n_nonfinite = 0, n_clamped = 0;
    __syncthreads();

    if (full && base + kQTile <= seg_end) {
        // whole tile inside one layer: one bias, LDS histogram
        const int bias = lay.bias[(uint64_t)u * lay.nseg + seg];
        const QConst qc = make_qconst(lay.E, lay.M, bias);
        const float gain = lay.gain[2 * ((uint64_t)u * lay.nseg + seg)], inv_gain = lay.gain[2 * ((uint64_t)u * lay.nseg + seg) + 1];
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const uint64_t i = base + (uint64_t)k * (kQThreads * 4) + threadIdx.x * 4;
            f4 eo;
            uint32_t packed = 0;
            Philox4 rw;
            if constexpr (kSR) rw = element_random_words(i, u, seed);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float v = __fadd_rn(gv[k][j], __fmul_rn(gamma, mv[k][j]));
                const float y = __fmul_rn(v, gain);   // real-valued scale: (1, 1) unless the plan carries one
                uint32_t s, flags;
                float q;
                if constexpr (kSR) quantize_stochastic(y, qc, lay.E, lay.M, bias, sign_shift, rw.w[j], s, q, flags);
                else quantize(y, qc, sign_shift, s, q, flags);
                q = __fmul_rn(q, inv_gain);
                eo[j] = (flags & 1u) ? 0.0f : __fsub_rn(v, q);
                n_nonfinite += flags & 1u;
                n_clamped += (flags >> 1) & 1u;
                packed |= s << (8 * j);
                atomicAdd(&h_lds[s * kHistRep + lane_rep], 1u);
            }
            __builtin_nontemporal_store(eo, reinterpret_cast<f4 *>(mo + i));
            *reinterpret_cast<uint32_t *>(su + i) = packed;
        }
        __syncthreads();
        uint64_t *hist_book = hist + (uint64_t)(book_base + lay.segs[seg].book) * lay.A;
        // chunk_hist (single-layer vectors only: a tile is then a chunk): this tile's own counts, from which the
        // chunk's coded size follows once the code is known, without another sweep over the symbols
        uint16_t *ch = chunk_hist ? chunk_hist + ((uint64_t)u * lay.nchunks + blockIdx.x) * lay.A : nullptr;
        for (uint32_t bin = threadIdx.x; bin < lay.A; bin += kQThreads) {
            uint32_t s = 0;
#pragma unroll
            for (int r = 0; r < kHistRep; ++r) s += h_lds[bin * kHistRep + ((r + bin) & (kHistRep - 1))];
            if (s) atomicAdd(reinterpret_cast<unsigned long long *>(hist_book + bin), (unsigned long long)s);
            if (ch) ch[bin] = (uint16_t)s;
        }
    } else {
        // ragged tail of the vector or a tile that crosses a layer boundary: element path
        for (int k = 0; k < 8; ++k) {
            const uint64_t i = base + (uint64_t)k * kQThreads + threadIdx.x;
            if (i >= d) break;
            uint32_t s_i = seg;
            while (i >= lay.segs[s_i + 1].offset) ++s_i;
            const int bias = lay.bias[(uint64_t)u * lay.nseg + s_i];
            const QConst qe = make_qconst(lay.E, lay.M, bias);
            const float v = __fadd_rn(gu[i], __fmul_rn(gamma, mu[i]));
            const float y = __fmul_rn(v, lay.gain[2 * ((uint64_t)u * lay.nseg + s_i)]);
            uint32_t s, flags;
            float q;
            if constexpr (kSR)
                quantize_stochastic(y, qe, lay.E, lay.M, bias, sign_shift, element_random_words(i, u, seed).w[i & 3u], s,
                                    q, flags);
            else quantize(y, qe, sign_shift, s, q, flags);
            q = __fmul_rn(q, lay.gain[2 * ((uint64_t)u * lay.nseg + s_i) + 1]);
            mo[i] = (flags & 1u) ? 0.0f : __fsub_rn(v, q);
            n_nonfinite += flags & 1u;
            n_clamped += (flags >> 1) & 1u;
            su[i] = (uint8_t)s;
            atomicAdd(reinterpret_cast<unsigned long long *>(
                          hist + (uint64_t)(book_base + lay.segs[s_i].book) * lay.A + s), 1ull);
            if (chunk_hist) atomicAdd(&h_lds[s * kHistRep], 1u);
        }
        if (chunk_hist) {  // wavefront-uniform; single-layer vectors only: this is the vector's ragged last tile
            __syncthreads();
            uint16_t *ch = chunk_hist + ((uint64_t)u * lay.nchunks + blockIdx.x) * lay.A;
            for (uint32_t bin = threadIdx.x; bin < lay.A; bin += kQThreads) ch[bin] = (uint16_t)h_lds[bin * kHistRep];
        }
    }
    if (n_nonfinite)
        atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_NONFINITE), (unsigned long long)n_nonfinite);
    if (n_clamped)
        atomicAdd(reinterpret_cast<unsigned long long *>(status + CO3_STAT_CLAMPED), (unsigned long long)n_clamped);
}

// hist[i] = sum over the kHistGlobalRep copies of hist_rep[r][i]
__global__ __launch_bounds__(256) void k_reduce_hist(const uint64_t *__restrict__ hist_rep, uint64_t *__restrict__ hist,
                                                    uint64_t n)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint64_t s = 0;
#pragma unroll 8
    for (int r = 0; r < kHistGlobalRep; ++r) s += hist_rep[(uint64_t)r * n + i];
    hist[i] = s;
}

// Fill kernel used instead of a memset node so that callers may capture the sequence in a graph.
__global__ void k_zero_u64(uint64_t *p, uint64_t n)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

hipError_t launch_zero_u64(uint64_t *p, uint64_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    ProfScope prof(K_ZERO, s);
    hipLaunchKernelGGL(k_zero_u64, dim3((uint32_t)((n + 255) / 256)), dim3(256), 0, s, p, n);
    return hipGetLastError();
}

hipError_t launch_reduce_hist(const uint64_t *hist_rep, uint64_t *hist, uint64_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    ProfScope prof(K_REDUCE_HIST, s);
    hipLaunchKernelGGL(k_reduce_hist, dim3((uint32_t)((n + 255) / 256)), dim3(256), 0, s, hist_rep, hist, n);
    return hipGetLastError();
}

hipError_t launch_quantize(const Layout &lay, const co3_encode_args &a, const EncodeWs &ws, hipStream_t s)
{
    if (lay.U == 0) return hipSuccess;
    const uint64_t ntiles = (lay.d + kQTile - 1) / kQTile;
    const uint64_t sym_stride = symbol_row_stride(lay.d);
    const size_t lds = (size_t)lay.A * kHistRep * sizeof(uint32_t);
    if (lay.d) {  // a vector without elements still gets its (all-zero) symbol counts from the fold below
        ProfScope prof(K_QUANTIZE, s);
        if (a.rounding == CO3_ROUND_STOCHASTIC)
            hipLaunchKernelGGL(k_quantize<true>, dim3((uint32_t)ntiles, lay.U), dim3(kQThreads), lds, s, lay, a.g, a.m,
                               a.m_out, a.symbols, sym_stride, a.row_stride, a.gamma, a.seed, ws.hist_rep, ws.chunk_hist, a.status);
        else
            hipLaunchKernelGGL(k_quantize<false>, dim3((uint32_t)ntiles, lay.U), dim3(kQThreads), lds, s, lay, a.g, a.m,
                               a.m_out, a.symbols, sym_stride, a.row_stride, a.gamma, a.seed, ws.hist_rep, ws.chunk_hist, a.status);
    }
    return launch_reduce_hist(ws.hist_rep, a.hist, (uint64_t)lay.nbooks * lay.A, s);
}

}  // namespace co3
