// E-step in direct form on the vector ALUs (Section 3.1: each w_i goes to the centroid minimising
// ||w_i - c||^2). Every (vector, centroid) distance is evaluated as sum_j (x_j - c_j)^2 in fp32, whose
// relative error is about (d+2) * 2^-24 of the distance itself, so the decision is exact outside
// ties far tighter than 1e-5 relative. This kernel is the reference E-step of the library: the
// matrix-core kernel falls back to it for the vectors it cannot decide safely.
//
// Mapping: one lane owns VPT vectors held in registers; centroid tiles are staged in LDS and read
// with wave-uniform addresses (an LDS broadcast), so one LDS read feeds 64 * VPT distance
// evaluations. Centroids are visited in ascending index with a strict "<", which yields the lowest
// index among equal distances.
#include "common.h"

namespace cc {

constexpr int kThreads = 256;

template <int D, int VPT, int TILE>
__global__ __launch_bounds__(kThreads) void assign_direct_kernel(const float* __restrict__ X, uint32_t N,
                                                                 const float* __restrict__ C, uint32_t K,
                                                                 uint32_t* __restrict__ idx, float* __restrict__ dmin,
                                                                 const uint32_t* __restrict__ gate,
                                                                 uint32_t gate_limit)
{
    __shared__ float4 tile[TILE * D / 4];
    if (gate != nullptr && *gate <= gate_limit) return;  // uniform over the grid

    const uint32_t base = blockIdx.x * (kThreads * VPT) + threadIdx.x;
    float x[VPT][D];
    float best[VPT];
    uint32_t arg[VPT];
#pragma unroll
    for (int v = 0; v < VPT; ++v) {
        const uint32_t i = base + v * kThreads;
        const uint32_t ic = i < N ? i : N - 1;  // out-of-range lanes recompute the last vector, never store
        load_row<D>(X + size_t(ic) * D, x[v]);
        best[v] = INFINITY;
        arg[v] = 0;
    }

    const float4* C4 = reinterpret_cast<const float4*>(C);
    for (uint32_t k0 = 0; k0 < K; k0 += TILE) {
        const uint32_t nk = min(uint32_t(TILE), K - k0);
        __syncthreads();
        for (uint32_t t = threadIdx.x; t < nk * (D / 4); t += kThreads) tile[t] = C4[size_t(k0) * (D / 4) + t];
        __syncthreads();
        for (uint32_t k = 0; k < nk; ++k) {
            float c[D];
            load_row<D>(reinterpret_cast<const float*>(tile + k * (D / 4)), c);
#pragma unroll
            for (int v = 0; v < VPT; ++v) {
                const float acc = direct_sqdist<D>(x[v], c);
                if (acc < best[v]) {
                    best[v] = acc;
                    arg[v] = k0 + k;
                }
            }
        }
    }

#pragma unroll
    for (int v = 0; v < VPT; ++v) {
        const uint32_t i = base + v * kThreads;
        if (i < N) {
            idx[i] = arg[v];
            if (dmin != nullptr) dmin[i] = best[v];
        }
    }
}

template <int D, int VPT, int TILE>
static hipError_t launch_t(const float* X, uint32_t N, const float* C, uint32_t K, uint32_t* idx, float* dmin,
                           const uint32_t* gate, uint32_t gate_limit, hipStream_t s, Profile* profile)
{
    const uint32_t blocks = (N + kThreads * VPT - 1) / (kThreads * VPT);
    ProfileScope scope(profile, kProfEstepDirect, s);
    hipLaunchKernelGGL((assign_direct_kernel<D, VPT, TILE>), dim3(blocks), dim3(kThreads), 0, s, X, N, C, K, idx, dmin,
                       gate, gate_limit);
    return hipGetLastError();
}

hipError_t launch_assign_direct(const float* X, uint32_t N, uint32_t d, const float* C, uint32_t K, uint32_t* idx,
                                float* dmin, const uint32_t* gate, uint32_t gate_limit, hipStream_t s, Profile* profile)
{
    switch (d) {
        case 4: return launch_t<4, 4, 1024>(X, N, C, K, idx, dmin, gate, gate_limit, s, profile);
        case 8: return launch_t<8, 2, 512>(X, N, C, K, idx, dmin, gate, gate_limit, s, profile);
        case 16: return launch_t<16, 1, 256>(X, N, C, K, idx, dmin, gate, gate_limit, s, profile);
        default: return hipErrorInvalidValue;
    }
}

// Objective: sum of dmin in fp64. Stage 1: a fixed grid of blocks, block b sums a fixed contiguous
// range with a fixed tree; stage 2: one block sums the partials in index order. The shape depends
// only on N, so the result is reproducible.
__global__ __launch_bounds__(kThreads) void reduce_dmin_kernel(const float* __restrict__ dmin, uint32_t N,
                                                               double* __restrict__ partials)
{
    __shared__ double red[kThreads];
    const uint64_t per = (uint64_t(N) + gridDim.x - 1) / gridDim.x;
    const uint64_t lo = per * blockIdx.x, hi = min(lo + per, uint64_t(N));
    double acc = 0.0;
    for (uint64_t i = lo + threadIdx.x; i < hi; i += kThreads) acc += double(dmin[i]);
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int off = kThreads / 2; off > 0; off >>= 1) {
        if (int(threadIdx.x) < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) partials[blockIdx.x] = red[0];
}

__global__ __launch_bounds__(kThreads) void reduce_partials_kernel(const double* __restrict__ partials, uint32_t n,
                                                                   double* __restrict__ out)
{
    __shared__ double red[kThreads];
    double acc = 0.0;
    for (uint32_t i = threadIdx.x; i < n; i += kThreads) acc += partials[i];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int off = kThreads / 2; off > 0; off >>= 1) {
        if (int(threadIdx.x) < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = red[0];
}

hipError_t launch_reduce_dmin(const float* dmin, uint32_t N, double* partials, uint32_t partial_slots, double* out,
                              hipStream_t s)
{
    const uint32_t blocks = partial_slots;
    hipLaunchKernelGGL(reduce_dmin_kernel, dim3(blocks), dim3(kThreads), 0, s, dmin, N, partials);
    hipLaunchKernelGGL(reduce_partials_kernel, dim3(1), dim3(kThreads), 0, s, partials, blocks, out);
    return hipGetLastError();
}

}  // namespace cc
