// Refinement stage of the matrix-core E-step (Section 3.1: the codes must be the true argmin).
// The scoring kernels list every vector whose decision fell inside their rounding guard band; here
// those vectors are re-decided in direct form, which is accurate to ~1e-6 relative of the distance
// itself, over every centroid that can still be the nearest.
#include <algorithm>

#include "common.h"

namespace cc {

constexpr int kThreads = 256;

// One wave per listed vector: the 64 lanes stride over the candidate range with coalesced row loads,
// each keeps its best (distance, centroid index) as one 64-bit key (distance bits << 32 | index; distances
// are non-negative, so the integer order is distance first, then the lower index), and a shuffle
// reduction picks the minimum. The candidate range is the whole codebook, or - for a norm-ordered run -
// the window of the vector's 512-vector tile, which provably contains the nearest centroid.
template <int D>
__global__ __launch_bounds__(kThreads) void refine_kernel(const float* __restrict__ X, uint32_t N,
                                                          const float* __restrict__ rows,
                                                          const uint32_t* __restrict__ row_ids, uint32_t K,
                                                          WsHeader* hdr, const uint32_t* __restrict__ refine_list,
                                                          uint32_t refine_cap, const uint2* __restrict__ windows,
                                                          uint32_t* __restrict__ idx, float* __restrict__ dmin,
                                                          long long* sums, uint32_t* counts, WsPersist* persist)
{
    const uint32_t count = hdr->refine_count;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        hdr->refined_vectors += count;
        hdr->assign_calls += 1;
        hdr->cmax_bits = 0;                               // the next E-step scans its own codebook
        if (persist != nullptr) persist->hint_valid = 1;  // idx (norm-ordered) is a usable hint from now on
    }
    if (count > refine_cap) return;  // overflow is handled by the full direct pass
    const int lane = threadIdx.x & 63;
    const uint32_t wave = (blockIdx.x * kThreads + threadIdx.x) >> 6, waves = gridDim.x * (kThreads / 64);
    const int fpe = fixed_point_exp(hdr->absmax_bits, N);
    for (uint32_t e = wave; e < count; e += waves) {
        const uint32_t i = refine_list[e];
        float x[D];
        load_row<D>(X + size_t(i) * D, x);
        const uint2* wl = windows != nullptr ? windows + size_t(i / kWinTile) * kWinStride : nullptr;
        const uint32_t nruns = wl != nullptr ? wl[0].x : 1u;
        // all runs of the list in one load (at most kWinSlots <= 64 of them, one per lane): a load per run inside the
        // loop below would put a trip to memory in front of every run
        static_assert(kWinSlots <= 64, "one run per lane");
        uint2 my_run = make_uint2(0u, 0u);
        if (wl != nullptr && uint32_t(lane) < nruns) my_run = wl[1 + lane];
        unsigned long long best = ~0ull;
        for (uint32_t r = 0; r < nruns; ++r) {
            uint32_t lo = 0, hi = K;
            if (wl != nullptr) {
                lo = min(kWinQuad * uint32_t(__builtin_amdgcn_readlane(int(my_run.x), int(r))), K);
                hi = min(kWinQuad * uint32_t(__builtin_amdgcn_readlane(int(my_run.y), int(r))), K);
            }
            constexpr int U = 4;  // independent row loads in flight per lane
            for (uint32_t p0 = lo + lane; p0 < hi; p0 += U * 64) {
                float c[U][D];
                uint32_t k[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const uint32_t pos = min(p0 + u * 64, hi - 1);
                    load_row<D>(rows + size_t(pos) * D, c[u]);
                    k[u] = row_ids != nullptr ? row_ids[pos] : pos;
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const unsigned long long v =
                        (static_cast<unsigned long long>(__float_as_uint(direct_sqdist<D>(x, c[u]))) << 32) | k[u];
                    if (p0 + u * 64 < hi) best = v < best ? v : best;
                }
            }
        }
        for (int off = 32; off > 0; off >>= 1) {
            const unsigned long long o = __shfl_xor(best, off, 64);
            best = o < best ? o : best;
        }
        if (lane == 0 && best != ~0ull) {
            const uint32_t k_new = uint32_t(best & 0xffffffffull), k_old = idx[i];
            if (sums != nullptr && k_new != k_old) {
                // the scoring kernel already added this vector to its provisional cluster: move it
                accumulate_vector<D>(x, k_old, sums, counts, fpe, -1);
                accumulate_vector<D>(x, k_new, sums, counts, fpe, +1);
            }
            idx[i] = k_new;
            dmin[i] = __uint_as_float(uint32_t(best >> 32));
        }
    }
}

hipError_t launch_refine(const float* X, uint32_t N, uint32_t d, const float* C, uint32_t K, uint32_t* idx,
                         const Workspace& w, bool fix_sums, bool norm_ordered, hipStream_t s)
{
    const float* rows = norm_ordered ? w.csorted : C;
    const uint32_t* row_ids = norm_ordered ? w.cperm : nullptr;
    const uint2* windows = norm_ordered ? w.windows : nullptr;
    long long* sums = fix_sums ? w.sums : nullptr;
    uint32_t* counts = fix_sums ? w.counts : nullptr;
    WsPersist* persist = norm_ordered ? w.persist : nullptr;
    const dim3 grid(2048), block(kThreads);
    switch (d) {
        case 4: hipLaunchKernelGGL(refine_kernel<4>, grid, block, 0, s, X, N, rows, row_ids, K, w.hdr, w.refine_list, w.refine_cap, windows, idx, w.dmin, sums, counts, persist); break;
        case 8: hipLaunchKernelGGL(refine_kernel<8>, grid, block, 0, s, X, N, rows, row_ids, K, w.hdr, w.refine_list, w.refine_cap, windows, idx, w.dmin, sums, counts, persist); break;
        case 16: hipLaunchKernelGGL(refine_kernel<16>, grid, block, 0, s, X, N, rows, row_ids, K, w.hdr, w.refine_list, w.refine_cap, windows, idx, w.dmin, sums, counts, persist); break;
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
