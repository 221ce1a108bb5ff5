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

template <int D>
struct VecRegs {
    float v[D];
};

template <int D, int VPT, int TILE>
__global__ __launch_bounds__(kThreads) void assign_direct_kernel(const float* __restrict__ X, uint32_t N,
                                                                 const float* __restrict__ C, uint32_t K,
                                                                 uint32_t* __restrict__ idx,
                                                                 double* __restrict__ partials)
{
    __shared__ float4 tile[TILE * D / 4];
    __shared__ double red[kThreads / 64];

    const uint32_t base = blockIdx.x * (kThreads * VPT) + threadIdx.x;
    float x[VPT][D];
    float best[VPT];
    uint32_t arg[VPT];
#pragma unroll
    for (int v = 0; v < VPT; ++v) {
        const uint32_t i = base + v * kThreads;
        const uint32_t ic = i < N ? i : N - 1;  // out-of-range lanes recompute the last vector, never store
        const float4* src = reinterpret_cast<const float4*>(X + size_t(ic) * D);
#pragma unroll
        for (int q = 0; q < D / 4; ++q) {
            float4 t = src[q];
            x[v][4 * q + 0] = t.x; x[v][4 * q + 1] = t.y; x[v][4 * q + 2] = t.z; x[v][4 * q + 3] = t.w;
        }
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
#pragma unroll
            for (int q = 0; q < D / 4; ++q) {
                float4 t = tile[k * (D / 4) + q];
                c[4 * q + 0] = t.x; c[4 * q + 1] = t.y; c[4 * q + 2] = t.z; c[4 * q + 3] = t.w;
            }
#pragma unroll
            for (int v = 0; v < VPT; ++v) {
                float t0 = x[v][0] - c[0];
                float acc = t0 * t0;
#pragma unroll
                for (int j = 1; j < D; ++j) {
                    float t = x[v][j] - c[j];
                    acc = fmaf(t, t, acc);
                }
                if (acc < best[v]) {
                    best[v] = acc;
                    arg[v] = k0 + k;
                }
            }
        }
    }

    double local = 0.0;
#pragma unroll
    for (int v = 0; v < VPT; ++v) {
        const uint32_t i = base + v * kThreads;
        if (i < N) {
            idx[i] = arg[v];
            local += double(best[v]);
        }
    }
    if (partials != nullptr) {
        // fixed-shape reduction: lanes of a wave by xor-shuffle, then the four waves in order
        for (int off = 32; off > 0; off >>= 1) local += __shfl_xor(local, off, 64);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = local;
        __syncthreads();
        if (threadIdx.x == 0) partials[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
    }
}

template <int D, int VPT, int TILE>
static hipError_t launch_t(const float* X, uint32_t N, const float* C, uint32_t K, uint32_t* idx, double* partials,
                           uint32_t* n_partials_out, hipStream_t s)
{
    const uint32_t blocks = (N + kThreads * VPT - 1) / (kThreads * VPT);
    if (n_partials_out) *n_partials_out = blocks;
    hipLaunchKernelGGL((assign_direct_kernel<D, VPT, TILE>), dim3(blocks), dim3(kThreads), 0, s, X, N, C, K, idx,
                       partials);
    return hipGetLastError();
}

hipError_t launch_assign_direct(const float* X, uint32_t N, uint32_t d, const float* C, uint32_t K, uint32_t* idx,
                                double* partials, uint32_t* n_partials_out, hipStream_t s)
{
    switch (d) {
        case 4: return launch_t<4, 4, 1024>(X, N, C, K, idx, partials, n_partials_out, s);
        case 8: return launch_t<8, 2, 512>(X, N, C, K, idx, partials, n_partials_out, s);
        case 16: return launch_t<16, 1, 256>(X, N, C, K, idx, partials, n_partials_out, s);
        default: return hipErrorInvalidValue;
    }
}

// Sums the per-block partial objectives in index order (one block, fixed tree) so that the result does
// not depend on scheduling.
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

hipError_t launch_reduce_partials(const double* partials, uint32_t n, double* out, hipStream_t s)
{
    hipLaunchKernelGGL(reduce_partials_kernel, dim3(1), dim3(kThreads), 0, s, partials, n, out);
    return hipGetLastError();
}

}  // namespace cc
