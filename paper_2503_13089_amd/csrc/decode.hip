// Reconstruction (Section 3.1; the gather codebook[code] of the paper's layer listing):
// out_i = c_{idx_i}. Pure data movement: 4 bytes of code in, 4*d bytes of weights out per vector,
// with the codebook (K*d*4 <= 4 MB) served from cache. Each lane moves 16-byte pieces; the output is
// written with streaming (non-temporal) stores since it is never re-read here.
#include <algorithm>

#include "common.h"

namespace cc {

constexpr int kThreads = 256;
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Each block moves kThreads * U consecutive 16-byte pieces. Measured on MI355X at d = 4, K = 65536: a plain
// fill of the output runs at 6.7 TB/s and fill + code read at 7.1 TB/s, but the 16-byte gathers hit 64
// different cache lines per wave instruction and the L1 looks up about one line per clock, which adds
// ~20 us per 11.3M vectors whatever the unroll factor or cache policy; U = 1 was the fastest variant.
template <int D, int U>
__global__ __launch_bounds__(kThreads) void decode_kernel(const f32x4* __restrict__ C4, uint32_t K,
                                                          const uint32_t* __restrict__ idx, uint64_t n_chunks,
                                                          f32x4* __restrict__ out4)
{
    constexpr int Q = D / 4;  // 16-byte pieces per vector
    const uint64_t base = uint64_t(blockIdx.x) * (kThreads * U) + threadIdx.x;
    uint32_t k[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint64_t t = min(base + uint64_t(u) * kThreads, n_chunks - 1);
        const uint32_t kk = idx[t / Q];
        k[u] = kk < K ? kk : K - 1;  // never read outside the codebook
    }
    f32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint64_t t = min(base + uint64_t(u) * kThreads, n_chunks - 1);
        v[u] = C4[size_t(k[u]) * Q + uint32_t(t % Q)];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint64_t t = base + uint64_t(u) * kThreads;
        if (t < n_chunks) __builtin_nontemporal_store(v[u], &out4[t]);
    }
}

__global__ __launch_bounds__(kThreads) void decode_scalar_kernel(const float* __restrict__ C, uint32_t K, uint32_t d,
                                                                 const uint32_t* __restrict__ idx, uint64_t n,
                                                                 float* __restrict__ out)
{
    const uint64_t t = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
    if (t >= n) return;
    const uint32_t kk = idx[t / d];
    const uint32_t k = kk < K ? kk : K - 1;  // never read outside the codebook
    __builtin_nontemporal_store(C[size_t(k) * d + uint32_t(t % d)], &out[t]);
}

hipError_t launch_decode(const float* C, uint32_t K, uint32_t d, const uint32_t* idx, uint64_t N, float* out,
                         hipStream_t s)
{
    constexpr int U = 1;
    const uint64_t n_chunks = N * (d / 4);
    const uint32_t blocks = uint32_t((n_chunks + kThreads * U - 1) / (kThreads * U));
    const f32x4* C4 = reinterpret_cast<const f32x4*>(C);
    f32x4* out4 = reinterpret_cast<f32x4*>(out);
    switch (d) {
        case 4: hipLaunchKernelGGL((decode_kernel<4, U>), dim3(blocks), dim3(kThreads), 0, s, C4, K, idx, n_chunks, out4); break;
        case 8: hipLaunchKernelGGL((decode_kernel<8, U>), dim3(blocks), dim3(kThreads), 0, s, C4, K, idx, n_chunks, out4); break;
        case 12: hipLaunchKernelGGL((decode_kernel<12, U>), dim3(blocks), dim3(kThreads), 0, s, C4, K, idx, n_chunks, out4); break;
        case 16: hipLaunchKernelGGL((decode_kernel<16, U>), dim3(blocks), dim3(kThreads), 0, s, C4, K, idx, n_chunks, out4); break;
        default: {
            // rows that are not whole 16-byte pieces: one float per lane
            const uint64_t n = N * d;
            hipLaunchKernelGGL(decode_scalar_kernel, dim3(uint32_t((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, C, K,
                               d, idx, n, out);
        }
    }
    return hipGetLastError();
}

__global__ __launch_bounds__(kThreads) void pad_rows_kernel(const float* __restrict__ in, uint64_t n_out, uint32_t d_in,
                                                            uint32_t d_out, float* __restrict__ out)
{
    const uint64_t t = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
    if (t >= n_out) return;
    const uint64_t i = t / d_out;
    const uint32_t j = uint32_t(t % d_out);
    out[t] = j < d_in ? in[i * d_in + j] : 0.0f;
}

__global__ __launch_bounds__(kThreads) void unpad_rows_kernel(const float* __restrict__ in, uint64_t n_out, uint32_t d_in,
                                                              uint32_t d_out, float* __restrict__ out)
{
    const uint64_t t = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
    if (t >= n_out) return;
    out[t] = in[(t / d_out) * d_in + t % d_out];
}

hipError_t launch_pad_rows(const float* in, uint32_t n, uint32_t d_in, uint32_t d_out, float* out, hipStream_t s)
{
    const uint64_t n_out = uint64_t(n) * d_out;
    hipLaunchKernelGGL(pad_rows_kernel, dim3(uint32_t((n_out + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, in, n_out,
                       d_in, d_out, out);
    return hipGetLastError();
}

hipError_t launch_unpad_rows(const float* in, uint32_t n, uint32_t d_in, uint32_t d_out, float* out, hipStream_t s)
{
    const uint64_t n_out = uint64_t(n) * d_out;
    hipLaunchKernelGGL(unpad_rows_kernel, dim3(uint32_t((n_out + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, in, n_out,
                       d_in, d_out, out);
    return hipGetLastError();
}

__global__ __launch_bounds__(kThreads) void copy_f32_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                            size_t n)
{
    const size_t i = size_t(blockIdx.x) * kThreads + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

hipError_t launch_copy_f32(const float* src, float* dst, size_t n, hipStream_t s)
{
    hipLaunchKernelGGL(copy_f32_kernel, dim3(uint32_t((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, src, dst, n);
    return hipGetLastError();
}

}  // namespace cc
