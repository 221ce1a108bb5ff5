// Codebook gradient with the order of the codes prepared once (Section 3.3: training moves the codebook only,
// the codes stay as the clustering left them). The plan lists, cluster by cluster, the positions whose code is
// that cluster; a backward pass then reads each gradient entry once, straight from the weight's gradient, and
// adds it up in a fixed order. Nothing of the clustering workspace is needed.
#include <algorithm>

#include "common.h"

namespace cc {
namespace {

constexpr int kThreads = 256;
constexpr uint32_t kPlanMagic = 0x6770316cu;
constexpr uint32_t kItem = 1024;  // members per work item: one wave, at most 16 steps

struct PlanHeader {
    uint32_t magic, n, K, n_items;
};

struct PlanView {
    PlanHeader* hdr;
    uint32_t* starts;        // [K + 1] first sorted position of each cluster; starts[K] = codes below K
    uint32_t* item_starts;   // [K + 1] first work item of each cluster
    uint32_t* order;         // [n] positions, by (code, position)
    uint32_t* item_cluster;  // [max items] cluster of each work item
    size_t bytes;
};

size_t max_items(uint64_t n, uint32_t K) { return size_t(K) + size_t(n / kItem) + 1; }

PlanView view(void* base, uint64_t n, uint32_t K)
{
    PlanView v;
    size_t off = 0;
    auto take = [&](size_t bytes) {  // base == nullptr: only the size is wanted
        char* p = base ? static_cast<char*>(base) + off : nullptr;
        off += align256(bytes);
        return p;
    };
    v.hdr = reinterpret_cast<PlanHeader*>(take(sizeof(PlanHeader)));
    v.starts = reinterpret_cast<uint32_t*>(take(size_t(K + 1) * 4));
    v.item_starts = reinterpret_cast<uint32_t*>(take(size_t(K + 1) * 4));
    v.order = reinterpret_cast<uint32_t*>(take(size_t(n) * 4));
    v.item_cluster = reinterpret_cast<uint32_t*>(take(max_items(n, K) * 4));
    v.bytes = off;
    return v;
}

__global__ __launch_bounds__(kThreads) void plan_init_kernel(const uint16_t* __restrict__ codes, uint32_t n,
                                                             uint16_t* __restrict__ keys, uint32_t* __restrict__ order)
{
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= n) return;
    keys[i] = codes[i];
    order[i] = i;
}

// starts[t] = number of codes below t (first position of cluster t in the sorted order), t = 0 .. K
__global__ __launch_bounds__(kThreads) void plan_starts_kernel(const uint16_t* __restrict__ sorted_keys, uint32_t n, uint32_t K,
                                                               uint32_t* __restrict__ starts)
{
    const uint32_t t = blockIdx.x * kThreads + threadIdx.x;
    if (t > K) return;
    uint32_t a = 0, b = n;
    while (a < b) {
        const uint32_t m = a + (b - a) / 2;
        if (uint32_t(sorted_keys[m]) >= t) b = m; else a = m + 1;
    }
    starts[t] = a;
}

// One workgroup: work items per cluster (a cluster of m members takes ceil(m / kItem)), their exclusive scan.
__global__ __launch_bounds__(1024) void plan_items_kernel(const uint32_t* __restrict__ starts, uint32_t n, uint32_t K,
                                                          uint32_t* __restrict__ item_starts, PlanHeader* hdr)
{
    __shared__ uint32_t wave_sum[16];
    __shared__ uint32_t carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (uint32_t k0 = 0; k0 < K; k0 += 1024) {
        const uint32_t k = k0 + threadIdx.x;
        const uint32_t c = k < K ? (starts[k + 1] - starts[k] + kItem - 1) / kItem : 0u;
        uint32_t incl = c;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t v = uint32_t(__shfl_up(int(incl), off, 64));
            if (lane >= off) incl += v;
        }
        if (lane == 63) wave_sum[wave] = incl;
        __syncthreads();
        uint32_t before = carry;
        for (int w = 0; w < wave; ++w) before += wave_sum[w];
        if (k < K) item_starts[k] = before + incl - c;
        __syncthreads();
        if (threadIdx.x == 1023) carry = before + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        item_starts[K] = carry;
        hdr->magic = kPlanMagic;
        hdr->n = n;
        hdr->K = K;
        hdr->n_items = carry;
    }
}

// One wave per cluster writes the cluster's number into its work items.
__global__ __launch_bounds__(kThreads) void plan_item_cluster_kernel(const uint32_t* __restrict__ item_starts, uint32_t K,
                                                                     uint32_t* __restrict__ item_cluster)
{
    const uint32_t k = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (k >= K) return;
    for (uint32_t it = item_starts[k] + (threadIdx.x & 63); it < item_starts[k + 1]; it += 64) item_cluster[it] = k;
}

template <int DT>
__device__ __forceinline__ float grad_at(const void* g, uint64_t i)
{
    if constexpr (DT == 0) return static_cast<const float*>(g)[i];
    else if constexpr (DT == 1) return float(static_cast<const _Float16*>(g)[i]);
    else return __uint_as_float(uint32_t(static_cast<const uint16_t*>(g)[i]) << 16);
}

template <int DT>
__device__ __forceinline__ float from16(uint32_t bits)
{
    if constexpr (DT == 1) return float(__builtin_bit_cast(_Float16, uint16_t(bits)));
    else return __uint_as_float(bits << 16);
}

__device__ __forceinline__ double wave_sum_fixed_order(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__device__ __forceinline__ bool plan_matches(const PlanHeader* hdr, uint32_t n, uint32_t K)
{
    return hdr->magic == kPlanMagic && hdr->n == n && hdr->K == K;
}

// One wave per work item: lane l adds members l, l + 64, ... of the item in fp64, then the lanes are added in a
// fixed tree. VEC: the g entries of a member are one aligned 8- or 16-byte piece (16-bit gradients, g = 4 or 8,
// out_features a multiple of g); otherwise entry by entry, cut at the row's end (padding columns have no gradient).
template <int DT, int G, bool VEC>
__global__ __launch_bounds__(kThreads) void grad_items_kernel(const void* __restrict__ grad, uint32_t out_features, uint32_t g,
                                                              uint32_t per_row, uint32_t n, uint32_t K,
                                                              const PlanHeader* __restrict__ hdr,
                                                              const uint32_t* __restrict__ starts,
                                                              const uint32_t* __restrict__ item_starts,
                                                              const uint32_t* __restrict__ order,
                                                              const uint32_t* __restrict__ item_cluster,
                                                              double* __restrict__ partial)
{
    if (!plan_matches(hdr, n, K)) return;
    const uint32_t it = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (it >= hdr->n_items) return;
    const int lane = threadIdx.x & 63;
    // The clamps below change nothing for a plan as cc_layer_grad_plan wrote it; they keep every access in
    // bounds should the caller's buffer have been overwritten since.
    const uint32_t k = item_cluster[it];
    if (k >= K) return;
    const uint32_t j1 = min(min(starts[k] + (it - item_starts[k] + 1) * kItem, starts[k + 1]), n);
    const uint32_t j0 = min(starts[k] + (it - item_starts[k]) * kItem, j1);
    double acc[G];
#pragma unroll
    for (int c = 0; c < G; ++c) acc[c] = 0.0;
#pragma unroll 4
    for (uint32_t j = j0 + lane; j < j1; j += 64) {
        const uint32_t p = min(order[j], n - 1);
        const uint32_t r = p / per_row, col = (p - r * per_row) * g;
        const uint64_t at = uint64_t(r) * out_features + col;
        if constexpr (VEC) {
            static_assert(DT != 0 && (G == 4 || G == 8), "16-bit pieces");
            uint32_t w[G / 2];
            if constexpr (G == 4) {
                const uint2 t = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(grad) + at);
                w[0] = t.x; w[1] = t.y;
            } else {
                const uint4 t = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(grad) + at);
                w[0] = t.x; w[1] = t.y; w[2] = t.z; w[3] = t.w;
            }
#pragma unroll
            for (int c = 0; c < G; ++c) acc[c] += double(from16<DT>((w[c / 2] >> (16 * (c & 1))) & 0xffffu));
        } else {
            const uint32_t valid = min(g, out_features - col);
#pragma unroll
            for (int c = 0; c < G; ++c)
                if (uint32_t(c) < valid) acc[c] += double(grad_at<DT>(grad, at + c));
        }
    }
#pragma unroll
    for (int c = 0; c < G; ++c) {
        const double t = wave_sum_fixed_order(acc[c]);
        if (lane == 0 && uint32_t(c) < g) partial[size_t(it) * g + c] = t;
    }
}

// One thread per codebook entry: the cluster's work items in order, one rounding to fp32. A plan that was not
// built for these (num_codes, K) gives NaN everywhere.
__global__ __launch_bounds__(kThreads) void grad_finish_kernel(const double* __restrict__ partial, uint32_t g, uint32_t n,
                                                               uint32_t K, uint32_t item_cap,
                                                               const PlanHeader* __restrict__ hdr,
                                                               const uint32_t* __restrict__ item_starts,
                                                               float* __restrict__ grad_codebook)
{
    const uint32_t t = blockIdx.x * kThreads + threadIdx.x;
    if (t >= K * g) return;
    if (!plan_matches(hdr, n, K)) {
        grad_codebook[t] = __uint_as_float(0x7fc00000u);
        return;
    }
    const uint32_t k = t / g, c = t - k * g;
    double s = 0.0;
    const uint32_t end = min(item_starts[k + 1], min(hdr->n_items, item_cap));
    for (uint32_t it = item_starts[k]; it < end; ++it) s += partial[size_t(it) * g + c];
    grad_codebook[t] = float(s);
}

template <int DT>
hipError_t grad_items_t(const void* grad, uint32_t out_features, uint32_t g, uint32_t per_row, uint32_t n, uint32_t K,
                        const PlanView& v, double* partial, hipStream_t s)
{
    const dim3 grid(uint32_t((max_items(n, K) + kThreads / 64 - 1) / (kThreads / 64)));
#define CC_GI(G, VEC)                                                                                                  \
    hipLaunchKernelGGL((grad_items_kernel<DT, G, VEC>), grid, dim3(kThreads), 0, s, grad, out_features, g, per_row, n, K, \
                       v.hdr, v.starts, v.item_starts, v.order, v.item_cluster, partial)
    if constexpr (DT != 0) {
        if (g == 4 && out_features % 4 == 0) { CC_GI(4, true); return hipGetLastError(); }
        if (g == 8 && out_features % 8 == 0) { CC_GI(8, true); return hipGetLastError(); }
    }
    if (g <= 4) CC_GI(4, false);
    else if (g <= 8) CC_GI(8, false);
    else CC_GI(16, false);
#undef CC_GI
    return hipGetLastError();
}

}  // namespace

size_t layer_grad_plan_bytes(uint64_t num_codes, uint32_t K) { return view(nullptr, num_codes, K).bytes; }

size_t layer_grad_plan_build_bytes(uint64_t num_codes)
{
    return 2 * align256(size_t(num_codes) * 2) + align256(size_t(num_codes) * 4) + align256(sort_hist_bytes(num_codes));
}

size_t layer_grad_planned_bytes(uint64_t num_codes, uint32_t K, uint32_t g) { return align256(max_items(num_codes, K) * g * 8); }

hipError_t launch_layer_grad_plan(const uint16_t* codes, uint32_t n, uint32_t K, void* plan, void* workspace, hipStream_t s)
{
    const PlanView v = view(plan, n, K);
    char* base = static_cast<char*>(workspace);
    uint16_t* keys_a = reinterpret_cast<uint16_t*>(base);
    uint16_t* keys_b = reinterpret_cast<uint16_t*>(base + align256(size_t(n) * 2));
    uint32_t* ids_b = reinterpret_cast<uint32_t*>(base + 2 * align256(size_t(n) * 2));
    uint32_t* hist = reinterpret_cast<uint32_t*>(base + 2 * align256(size_t(n) * 2) + align256(size_t(n) * 4));
    hipLaunchKernelGGL(plan_init_kernel, dim3((n + kThreads - 1) / kThreads), dim3(kThreads), 0, s, codes, n, keys_a, v.order);
    if (hipError_t e = launch_sort_u16(keys_a, v.order, keys_b, ids_b, n, hist, s); e != hipSuccess) return e;
    hipLaunchKernelGGL(plan_starts_kernel, dim3((K + 1 + kThreads - 1) / kThreads), dim3(kThreads), 0, s, keys_a, n, K, v.starts);
    hipLaunchKernelGGL(plan_items_kernel, dim3(1), dim3(1024), 0, s, v.starts, n, K, v.item_starts, v.hdr);
    hipLaunchKernelGGL(plan_item_cluster_kernel, dim3((K + kThreads / 64 - 1) / (kThreads / 64)), dim3(kThreads), 0, s,
                       v.item_starts, K, v.item_cluster);
    return hipGetLastError();
}

hipError_t launch_layer_grad_planned(const void* grad, int dtype, uint32_t in_features, uint32_t out_features, uint32_t K,
                                     uint32_t g, uint32_t n, const void* plan, float* grad_codebook, void* workspace,
                                     hipStream_t s)
{
    (void)in_features;
    const PlanView v = view(const_cast<void*>(plan), n, K);
    const uint32_t per_row = (out_features + g - 1) / g;
    double* partial = static_cast<double*>(workspace);
    hipError_t e;
    switch (dtype) {
        case 0: e = grad_items_t<0>(grad, out_features, g, per_row, n, K, v, partial, s); break;
        case 1: e = grad_items_t<1>(grad, out_features, g, per_row, n, K, v, partial, s); break;
        case 2: e = grad_items_t<2>(grad, out_features, g, per_row, n, K, v, partial, s); break;
        default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    const uint32_t entries = K * g;  // K <= 65536, g <= 16
    hipLaunchKernelGGL(grad_finish_kernel, dim3((entries + kThreads - 1) / kThreads), dim3(kThreads), 0, s, partial, g, n, K,
                       uint32_t(max_items(n, K)), v.hdr, v.item_starts, grad_codebook);
    return hipGetLastError();
}

}  // namespace cc
