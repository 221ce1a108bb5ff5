// Refinement stage of the matrix-core E-step (Section 3.1: the codes must be the true argmin).
// The scoring kernels list every vector whose decision fell inside their rounding guard band; here
// those vectors are re-decided over ALL K centroids in direct form, which is accurate to ~1e-6
// relative of the distance itself.
#include <algorithm>

#include "common.h"

namespace cc {

constexpr int kThreads = 256;

// Work item =
// (chunk of 64 listed vectors, slice of the codebook); each lane keeps the best (distance, index) of
// its slice and merges it with a 64-bit atomicMin on (distance bits << 32 | index): distances are
// non-negative, so the integer order is (distance, then lowest index) - order independent.
template <int D>
__global__ __launch_bounds__(64) void refine_kernel(const float* __restrict__ X, const float* __restrict__ C,
                                                    uint32_t K, const WsHeader* __restrict__ hdr,
                                                    const uint32_t* __restrict__ refine_list,
                                                    unsigned long long* __restrict__ refine_best,
                                                    uint32_t refine_cap, uint32_t slices)
{
    const uint32_t count = hdr->refine_count;
    if (count == 0 || count > refine_cap) return;  // overflow is handled by the full direct pass
    const uint32_t chunks = (count + 63) / 64;
    const uint32_t per = (K + slices - 1) / slices;
    for (uint32_t w = blockIdx.x; w < chunks * slices; w += gridDim.x) {
        const uint32_t chunk = w / slices, slice = w % slices;
        const uint32_t e = chunk * 64 + threadIdx.x;
        const uint32_t ec = min(e, count - 1);
        float x[D];
        load_row<D>(X + size_t(refine_list[ec]) * D, x);
        const uint32_t k_lo = slice * per, k_hi = min(k_lo + per, K);
        float bd = INFINITY;
        uint32_t bk = 0;
        // k is wave-uniform: a centroid is fetched once per wave; four fetches are in flight at a time
        uint32_t k = k_lo;
        for (; k + 4 <= k_hi; k += 4) {
            float c[4][D];
#pragma unroll
            for (int u = 0; u < 4; ++u) load_row<D>(C + size_t(k + u) * D, c[u]);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float dk = direct_sqdist<D>(x, c[u]);
                if (dk < bd) {
                    bd = dk;
                    bk = k + u;
                }
            }
        }
        for (; k < k_hi; ++k) {
            float c[D];
            load_row<D>(C + size_t(k) * D, c);
            const float dk = direct_sqdist<D>(x, c);
            if (dk < bd) {
                bd = dk;
                bk = k;
            }
        }
        if (e < count && k_lo < k_hi)
            atomicMin(&refine_best[e], (static_cast<unsigned long long>(__float_as_uint(bd)) << 32) | bk);
    }
}

template <int D>
__global__ __launch_bounds__(kThreads) void refine_finish_kernel(WsHeader* hdr, const uint32_t* __restrict__ refine_list,
                                                                 const unsigned long long* __restrict__ refine_best,
                                                                 uint32_t refine_cap, uint32_t* __restrict__ idx,
                                                                 float* __restrict__ dmin, const float* __restrict__ X,
                                                                 uint32_t N, long long* sums, uint32_t* counts,
                                                                 WsPersist* persist)
{
    const uint32_t count = hdr->refine_count;
    const uint32_t e = blockIdx.x * kThreads + threadIdx.x;
    if (e == 0) {
        if (persist != nullptr) persist->hint_valid = 1;  // idx (norm-ordered) is a usable hint from now on
        hdr->refined_vectors += count;
        hdr->assign_calls += 1;
        hdr->cmax_bits = 0;  // the next E-step scans its own codebook
    }
    if (count > refine_cap) return;
    const int fpe = fixed_point_exp(hdr->absmax_bits, N);
    for (uint32_t j = e; j < count; j += gridDim.x * kThreads) {
        const unsigned long long v = refine_best[j];
        const uint32_t i = refine_list[j];
        const uint32_t k_new = uint32_t(v & 0xffffffffull), k_old = idx[i];
        if (sums != nullptr && k_new != k_old) {
            // the scoring kernel already added this vector to its provisional cluster: move it
            float x[D];
            load_row<D>(X + size_t(i) * D, x);
            accumulate_vector<D>(x, k_old, sums, counts, fpe, -1);
            accumulate_vector<D>(x, k_new, sums, counts, fpe, +1);
        }
        idx[i] = k_new;
        dmin[i] = __uint_as_float(uint32_t(v >> 32));
    }
}

template <int D>
static void launch_refine_t(const float* X, uint32_t N, const float* C, uint32_t K, uint32_t* idx, const Workspace& w,
                            bool fix_sums, bool mark_hint, uint32_t slices, hipStream_t s)
{
    hipLaunchKernelGGL(refine_kernel<D>, dim3(4096), dim3(64), 0, s, X, C, K, w.hdr, w.refine_list, w.refine_best,
                       w.refine_cap, slices);
    hipLaunchKernelGGL(refine_finish_kernel<D>, dim3(256), dim3(kThreads), 0, s, w.hdr, w.refine_list, w.refine_best,
                       w.refine_cap, idx, w.dmin, X, N, fix_sums ? w.sums : nullptr, fix_sums ? w.counts : nullptr,
                       mark_hint ? w.persist : nullptr);
}

hipError_t launch_refine(const float* X, uint32_t N, uint32_t d, const float* C, uint32_t K, uint32_t* idx,
                         const Workspace& w, bool fix_sums, bool mark_hint, hipStream_t s)
{
    const uint32_t slices = std::max(1u, std::min(128u, K / 512));
    switch (d) {
        case 4: launch_refine_t<4>(X, N, C, K, idx, w, fix_sums, mark_hint, slices, s); break;
        case 8: launch_refine_t<8>(X, N, C, K, idx, w, fix_sums, mark_hint, slices, s); break;
        case 16: launch_refine_t<16>(X, N, C, K, idx, w, fix_sums, mark_hint, slices, s); break;
        default: return hipErrorInvalidValue;
    }
    // overflow path: more guard-band vectors than the list holds -> decide everything in direct form
    // (and rebuild the cluster sums from those codes)
    hipError_t e = launch_assign_direct(X, N, d, C, K, idx, w.dmin, &w.hdr->refine_count, w.refine_cap, s);
    if (e != hipSuccess) return e;
    if (fix_sums) {
        e = launch_zero_accumulators(w, K, d, &w.hdr->refine_count, w.refine_cap, s);
        if (e != hipSuccess) return e;
        e = launch_accumulate(X, N, d, idx, K, w, &w.hdr->refine_count, w.refine_cap, s);
        if (e != hipSuccess) return e;
    }
    return hipGetLastError();
}

}  // namespace cc
