// Refinement stage of the matrix-core E-step (Section 3.1: the codes must be the true argmin).
// The scoring kernels list every vector whose decision fell inside their rounding guard band; here
// those vectors are re-decided over ALL K centroids in direct form, which is accurate to ~1e-6
// relative of the distance itself.
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
        for (uint32_t k = k_lo; k < k_hi; ++k) {  // k is wave-uniform: the centroid is fetched once per wave
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

__global__ __launch_bounds__(kThreads) void refine_finish_kernel(WsHeader* hdr, const uint32_t* __restrict__ refine_list,
                                                                 const unsigned long long* __restrict__ refine_best,
                                                                 uint32_t refine_cap, uint32_t* __restrict__ idx,
                                                                 float* __restrict__ dmin)
{
    const uint32_t count = hdr->refine_count;
    const uint32_t e = blockIdx.x * kThreads + threadIdx.x;
    if (e == 0) {
        hdr->refined_vectors += count;
        hdr->assign_calls += 1;
    }
    if (count > refine_cap) return;
    for (uint32_t j = e; j < count; j += gridDim.x * kThreads) {
        const unsigned long long v = refine_best[j];
        const uint32_t i = refine_list[j];
        idx[i] = uint32_t(v & 0xffffffffull);
        dmin[i] = __uint_as_float(uint32_t(v >> 32));
    }
}


hipError_t launch_refine(const float* X, uint32_t N, uint32_t d, const float* C, uint32_t K, uint32_t* idx,
                         const Workspace& w, hipStream_t s)
{
    const uint32_t slices = K >= 4096 ? 32 : (K >= 256 ? 4 : 1);
    switch (d) {
        case 4: hipLaunchKernelGGL(refine_kernel<4>, dim3(4096), dim3(64), 0, s, X, C, K, w.hdr, w.refine_list, w.refine_best, w.refine_cap, slices); break;
        case 8: hipLaunchKernelGGL(refine_kernel<8>, dim3(4096), dim3(64), 0, s, X, C, K, w.hdr, w.refine_list, w.refine_best, w.refine_cap, slices); break;
        case 16: hipLaunchKernelGGL(refine_kernel<16>, dim3(4096), dim3(64), 0, s, X, C, K, w.hdr, w.refine_list, w.refine_best, w.refine_cap, slices); break;
        default: return hipErrorInvalidValue;
    }
    hipLaunchKernelGGL(refine_finish_kernel, dim3(256), dim3(kThreads), 0, s, w.hdr, w.refine_list, w.refine_best,
                       w.refine_cap, idx, w.dmin);
    // overflow path: more guard-band vectors than the list holds -> decide everything in direct form
    hipError_t e = launch_assign_direct(X, N, d, C, K, idx, w.dmin, &w.hdr->refine_count, w.refine_cap, s);
    if (e != hipSuccess) return e;
    return hipGetLastError();
}

}  // namespace cc
