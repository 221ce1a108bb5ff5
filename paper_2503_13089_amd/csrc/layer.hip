// Data movement of the compressed linear layer (Section 3.1 footnote, Section 3.2, the paper's layer
// listing): the reshape that produces the vectors to cluster, the 16-bit storage formats, and the
// reconstruction of the weight from (codebook, codes) with the padding columns cut off.
#include "common.h"

namespace cc {

constexpr int kThreads = 256;

// ---- element conversions -----------------------------------------------------------------------
// bf16 is the upper half of the fp32 pattern; rounding to nearest even adds 0x7fff + (lowest kept bit).
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float v)
{
    const uint32_t b = __float_as_uint(v);
    if ((b & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;  // NaN
    return uint16_t((b + 0x7fffu + ((b >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t h) { return __uint_as_float(uint32_t(h) << 16); }
__device__ __forceinline__ uint16_t f32_to_f16_bits(float v)
{
    const _Float16 h = _Float16(v);  // round to nearest even
    return *reinterpret_cast<const uint16_t*>(&h);
}
__device__ __forceinline__ float f16_bits_to_f32(uint16_t b) { return float(*reinterpret_cast<const _Float16*>(&b)); }

template <int DT>
__device__ __forceinline__ float load_as_f32(const void* p, size_t i)
{
    if constexpr (DT == 0) return static_cast<const float*>(p)[i];
    else if constexpr (DT == 1) return f16_bits_to_f32(static_cast<const uint16_t*>(p)[i]);
    else return bf16_bits_to_f32(static_cast<const uint16_t*>(p)[i]);
}

// ---- vectors to cluster: transpose [out, in] -> [in, out + deficiency] with zero padding, as fp32.
// 64 x 64 tiles through LDS so that both the reads (along in) and the writes (along out) are contiguous.
template <int DT>
__global__ __launch_bounds__(kThreads) void layer_vectors_kernel(const void* __restrict__ weight, uint32_t out_features,
                                                                 uint32_t in_features, uint32_t width,
                                                                 float* __restrict__ vectors)
{
    __shared__ float tile[64][65];
    const uint32_t c0 = blockIdx.x * 64;  // first out-feature (column of the transpose) of this tile
    const uint32_t r0 = blockIdx.y * 64;  // first in-feature (row of the transpose)
    const uint32_t tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (uint32_t j = ty; j < 64; j += 4) {  // weight rows c0 + j, columns r0 + tx
        const uint32_t c = c0 + j, r = r0 + tx;
        tile[j][tx] = (c < out_features && r < in_features) ? load_as_f32<DT>(weight, size_t(c) * in_features + r) : 0.0f;
    }
    __syncthreads();
    for (uint32_t j = ty; j < 64; j += 4) {  // transposed rows r0 + j, columns c0 + tx (padding columns get the zeros)
        const uint32_t r = r0 + j, c = c0 + tx;
        if (r < in_features && c < width) vectors[size_t(r) * width + c] = tile[tx][j];
    }
}

hipError_t launch_layer_vectors(const void* weight, int dtype, uint32_t out_features, uint32_t in_features, uint32_t g,
                                float* vectors, hipStream_t s)
{
    const uint32_t width = (out_features + g - 1) / g * g;
    const dim3 grid((width + 63) / 64, (in_features + 63) / 64);
    switch (dtype) {
        case 0: hipLaunchKernelGGL(layer_vectors_kernel<0>, grid, dim3(kThreads), 0, s, weight, out_features, in_features, width, vectors); break;
        case 1: hipLaunchKernelGGL(layer_vectors_kernel<1>, grid, dim3(kThreads), 0, s, weight, out_features, in_features, width, vectors); break;
        case 2: hipLaunchKernelGGL(layer_vectors_kernel<2>, grid, dim3(kThreads), 0, s, weight, out_features, in_features, width, vectors); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ---- storage formats
template <int DT>
__global__ __launch_bounds__(kThreads) void pack_codebook_kernel16(const float* __restrict__ in, size_t n,
                                                                  uint16_t* __restrict__ out)
{
    const size_t i = size_t(blockIdx.x) * kThreads + threadIdx.x;
    if (i < n) out[i] = DT == 1 ? f32_to_f16_bits(in[i]) : f32_to_bf16_bits(in[i]);
}

hipError_t launch_layer_pack_codebook(const float* centroids, size_t n, void* codebook, int dtype, hipStream_t s)
{
    const dim3 grid(uint32_t((n + kThreads - 1) / kThreads));
    uint16_t* out = static_cast<uint16_t*>(codebook);
    switch (dtype) {
        case 1: hipLaunchKernelGGL(pack_codebook_kernel16<1>, grid, dim3(kThreads), 0, s, centroids, n, out); break;
        case 2: hipLaunchKernelGGL(pack_codebook_kernel16<2>, grid, dim3(kThreads), 0, s, centroids, n, out); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

__global__ __launch_bounds__(kThreads) void pack_codes_kernel(const uint32_t* __restrict__ idx, uint64_t n, uint32_t K,
                                                              uint16_t* __restrict__ codes)
{
    const uint64_t i = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
    if (i < n) codes[i] = uint16_t(min(idx[i], K - 1));
}

hipError_t launch_layer_pack_codes(const uint32_t* idx, uint64_t n, uint32_t K, uint16_t* codes, hipStream_t s)
{
    hipLaunchKernelGGL(pack_codes_kernel, dim3(uint32_t((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, idx, n, K,
                       codes);
    return hipGetLastError();
}

// ---- reconstruction: one lane per code; its g elements go to weight[r][c .. c + g) minus the padding.
// T is the element's storage type (2 or 4 bytes). Lanes of a wave write neighbouring pieces of one row.
template <typename T>
__global__ __launch_bounds__(kThreads) void layer_weight_kernel(const T* __restrict__ codebook, uint32_t K, uint32_t g,
                                                                const uint16_t* __restrict__ codes, uint64_t num_codes,
                                                                uint32_t per_row, uint32_t out_features,
                                                                T* __restrict__ weight)
{
    const uint64_t v = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
    if (v >= num_codes) return;
    const uint32_t r = uint32_t(v / per_row), c = uint32_t(v % per_row) * g;
    const uint32_t k = min(uint32_t(codes[v]), K - 1);  // never read outside the codebook
    const T* row = codebook + size_t(k) * g;
    T* dst = weight + size_t(r) * out_features + c;
    const uint32_t n = min(g, out_features - c);  // c < out_features always: at most g - 1 padding columns
    for (uint32_t j = 0; j < n; ++j) dst[j] = row[j];
}

// g = 4 or 8 with no padding and 16-bit elements: whole rows as one 8- or 16-byte piece
template <typename V>
__global__ __launch_bounds__(kThreads) void layer_weight_vec_kernel(const V* __restrict__ codebook, uint32_t K,
                                                                    const uint16_t* __restrict__ codes,
                                                                    uint64_t num_codes, V* __restrict__ weight)
{
    const uint64_t v = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
    if (v >= num_codes) return;
    const uint32_t k = min(uint32_t(codes[v]), K - 1);
    __builtin_nontemporal_store(codebook[k], &weight[v]);
}

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

hipError_t launch_layer_weight(const void* codebook, int dtype, uint32_t K, uint32_t g, const uint16_t* codes,
                               uint32_t in_features, uint32_t out_features, void* weight, hipStream_t s)
{
    const uint32_t per_row = (out_features + g - 1) / g;
    const uint64_t num_codes = uint64_t(in_features) * per_row;
    const dim3 grid(uint32_t((num_codes + kThreads - 1) / kThreads));
    const bool whole = out_features % g == 0;
    if (dtype != 0 && whole && g == 4) {
        hipLaunchKernelGGL(layer_weight_vec_kernel<u32x2>, grid, dim3(kThreads), 0, s, static_cast<const u32x2*>(codebook), K,
                           codes, num_codes, static_cast<u32x2*>(weight));
    } else if (dtype != 0 && whole && g == 8) {
        hipLaunchKernelGGL(layer_weight_vec_kernel<u32x4>, grid, dim3(kThreads), 0, s, static_cast<const u32x4*>(codebook), K,
                           codes, num_codes, static_cast<u32x4*>(weight));
    } else if (dtype == 0) {
        hipLaunchKernelGGL(layer_weight_kernel<uint32_t>, grid, dim3(kThreads), 0, s, static_cast<const uint32_t*>(codebook),
                           K, g, codes, num_codes, per_row, out_features, static_cast<uint32_t*>(weight));
    } else {
        hipLaunchKernelGGL(layer_weight_kernel<uint16_t>, grid, dim3(kThreads), 0, s, static_cast<const uint16_t*>(codebook),
                           K, g, codes, num_codes, per_row, out_features, static_cast<uint16_t*>(weight));
    }
    return hipGetLastError();
}

// ---- codebook gradient, first step: the gradient of the weight as fp32 vectors in the layout of the
// clustering (padding columns and padding components zero), and the codes widened for the M-step kernels.
template <int DT>
__global__ __launch_bounds__(kThreads) void layer_grad_vectors_kernel(const void* __restrict__ grad, uint32_t out_features,
                                                                      uint32_t width, uint32_t g, uint32_t d_pad,
                                                                      const uint16_t* __restrict__ codes,
                                                                      uint64_t num_codes, float* __restrict__ vectors,
                                                                      uint32_t* __restrict__ idx)
{
    const uint64_t t = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
    if (t >= num_codes * d_pad) return;
    const uint64_t v = t / d_pad;
    const uint32_t j = uint32_t(t % d_pad);
    float val = 0.0f;
    if (j < g) {
        const uint64_t flat = v * g + j;  // position in the padded transpose
        const uint64_t r = flat / width;
        const uint32_t c = uint32_t(flat % width);
        if (c < out_features) val = load_as_f32<DT>(grad, r * out_features + c);
    }
    vectors[t] = val;
    if (j == 0) idx[v] = codes[v];
}

hipError_t launch_layer_grad_vectors(const void* grad, int dtype, uint32_t in_features, uint32_t out_features,
                                     uint32_t g, uint32_t d_pad, const uint16_t* codes, uint64_t num_codes, float* vectors,
                                     uint32_t* idx, hipStream_t s)
{
    (void)in_features;
    const uint32_t width = (out_features + g - 1) / g * g;
    const uint64_t n = num_codes * d_pad;
    const dim3 grid(uint32_t((n + kThreads - 1) / kThreads));
    switch (dtype) {
        case 0: hipLaunchKernelGGL(layer_grad_vectors_kernel<0>, grid, dim3(kThreads), 0, s, grad, out_features, width, g, d_pad, codes, num_codes, vectors, idx); break;
        case 1: hipLaunchKernelGGL(layer_grad_vectors_kernel<1>, grid, dim3(kThreads), 0, s, grad, out_features, width, g, d_pad, codes, num_codes, vectors, idx); break;
        case 2: hipLaunchKernelGGL(layer_grad_vectors_kernel<2>, grid, dim3(kThreads), 0, s, grad, out_features, width, g, d_pad, codes, num_codes, vectors, idx); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace cc
