// M-step (Section 3.1): c_k <- mean of the vectors assigned to cluster k.
//
// The cluster sums are accumulated as 64-bit integers: each input is scaled by 2^e and rounded to
// an integer, with e chosen from the largest input magnitude M and from N so that N terms of size
// <= M * 2^e cannot overflow 62 bits. Integer addition is associative, so the sums - and with them
// the centroids - do not depend on the order in which the atomics land: same inputs, same bits.
// For fp16-representable inputs (multiples of 2^-24) and e >= 24 the sums are exact.
//
// An empty cluster keeps its previous centroid (the paper does not say what the mean of no vectors is).
#include <algorithm>

#include "common.h"

namespace cc {

constexpr int kThreads = 256;

__global__ void reset_header_kernel(WsHeader* hdr)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        hdr->absmax_bits = 0;
        hdr->refine_count = 0;
        hdr->x_not_f16 = 0;
        hdr->cmax_bits = 0;
        hdr->refined_vectors = 0;
        hdr->skipped_vectors = 0;
        hdr->assign_calls = 0;
        hdr->window_stages = 0;
        hdr->window_total = 0;
        hdr->fixed_point_exp = 0;
        hdr->x_nonfinite = 0;
    }
}

hipError_t launch_reset_header(WsHeader* hdr, hipStream_t s)
{
    hipLaunchKernelGGL(reset_header_kernel, dim3(1), dim3(64), 0, s, hdr);
    return hipGetLastError();
}

__global__ void bump_assign_calls_kernel(WsHeader* hdr)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) hdr->assign_calls += 1;
}

hipError_t launch_bump_assign_calls(WsHeader* hdr, hipStream_t s)
{
    hipLaunchKernelGGL(bump_assign_calls_kernel, dim3(1), dim3(64), 0, s, hdr);
    return hipGetLastError();
}

// One pass over the inputs: max |x| over the finite inputs as the maximum of the (sign-cleared) fp32 bit patterns
// (for finite floats the integer order of the patterns is the order of the magnitudes), whether any input is Inf
// or NaN (the caller's precondition is that none is; such a component is left out of the cluster sums and the
// fact is reported in the statistics), and whether the vectors qualify
// for the fp16 matrix-core kernels: |x| < 2^15, and every value of the fp16 normal range (|x| >= 2^-14)
// survives a round trip through fp16 (then -2x is also an fp16 number). Smaller values need not be fp16
// numbers - bf16 weights have many that are not: what their fp16 rounding loses is at most 2^-25 each, which
// those kernels add to their guard band per vector.
__global__ __launch_bounds__(kThreads) void scan_inputs_kernel(const float4* __restrict__ X4, uint64_t n4, WsHeader* hdr)
{
    __shared__ uint32_t red_m[kThreads / 64], red_f[kThreads / 64];
    uint32_t m = 0, bad = 0;  // bad: bit 0 = not fit for the fp16 kernels, bit 1 = a non-finite input
    for (uint64_t i = uint64_t(blockIdx.x) * kThreads + threadIdx.x; i < n4; i += uint64_t(gridDim.x) * kThreads) {
        const float4 t = X4[i];
        const float v[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t a = __float_as_uint(v[j]) & 0x7fffffffu;
            const bool finite = a < 0x7f800000u;
            m = finite ? max(m, a) : m;
            const float back = float(_Float16(v[j]));
            bad |= uint32_t((back != v[j] && a >= 0x38800000u /* 2^-14 */) || (a >= 0x47000000u /* 2^15 */)) |
                   (finite ? 0u : 2u);
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        m = max(m, uint32_t(__shfl_xor(int(m), off, 64)));
        bad |= uint32_t(__shfl_xor(int(bad), off, 64));
    }
    if ((threadIdx.x & 63) == 0) {
        red_m[threadIdx.x >> 6] = m;
        red_f[threadIdx.x >> 6] = bad;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kThreads / 64; ++w) {
            m = max(m, red_m[w]);
            bad |= red_f[w];
        }
        // most blocks see nothing new: a (possibly stale) look at the running maximum spares the memory-side atomic,
        // 2048 of which on one address cost as much as a third of the scan
        if (m > __builtin_nontemporal_load(&hdr->absmax_bits)) atomicMax(&hdr->absmax_bits, m);
        if (bad & 1u) atomicOr(&hdr->x_not_f16, 1u);
        if (bad & 2u) atomicOr(&hdr->x_nonfinite, 1u);
    }
}

hipError_t launch_scan_inputs(const float* X, uint64_t n_floats, WsHeader* hdr, hipStream_t s)
{
    const uint64_t n4 = n_floats / 4;  // d is a multiple of 4
    const uint32_t blocks = uint32_t(std::min<uint64_t>((n4 + kThreads - 1) / kThreads, 2048));
    hipLaunchKernelGGL(scan_inputs_kernel, dim3(blocks), dim3(kThreads), 0, s, reinterpret_cast<const float4*>(X), n4,
                       hdr);
    return hipGetLastError();
}

// The same scan for rows of 16-bit numbers (DT 1 = fp16, 2 = bf16; a layer's gradient), four numbers per step: the
// largest finite magnitude, as the bits of its fp32 value, and whether any number is Inf or NaN. Magnitudes of one
// 16-bit format order like their bit patterns, so the conversion happens once, at the end.
template <int DT>
__global__ __launch_bounds__(kThreads) void scan_inputs16_kernel(const uint2* __restrict__ X2, uint64_t n2, WsHeader* hdr)
{
    __shared__ uint32_t red_m[kThreads / 64], red_f[kThreads / 64];
    constexpr uint32_t kInf = DT == 1 ? 0x7c00u : 0x7f80u;
    uint32_t m = 0, bad = 0;
    const auto look = [&](uint32_t w) {
        const uint32_t lo = w & 0x7fffu, hi = (w >> 16) & 0x7fffu;
        m = lo < kInf ? max(m, lo) : m;
        m = hi < kInf ? max(m, hi) : m;
        bad |= (lo < kInf && hi < kInf) ? 0u : 1u;
    };
    // 16 bytes per load, four loads in flight per thread; X2 is 16-byte aligned whenever it holds a whole uint4
    const uint4* X4 = reinterpret_cast<const uint4*>(X2);
    const uint64_t n4 = n2 / 2, stride = uint64_t(gridDim.x) * kThreads;
    uint64_t i = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
    for (; i + 3 * stride < n4; i += 4 * stride) {
        uint4 t[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) t[u] = X4[i + u * stride];
#pragma unroll
        for (int u = 0; u < 4; ++u) { look(t[u].x); look(t[u].y); look(t[u].z); look(t[u].w); }
    }
    for (; i < n4; i += stride) {
        const uint4 t = X4[i];
        look(t.x); look(t.y); look(t.z); look(t.w);
    }
    if ((n2 & 1) && blockIdx.x == 0 && threadIdx.x == 0) {  // four numbers left over
        const uint2 t = X2[n2 - 1];
        look(t.x); look(t.y);
    }
    for (int off = 32; off > 0; off >>= 1) {
        m = max(m, uint32_t(__shfl_xor(int(m), off, 64)));
        bad |= uint32_t(__shfl_xor(int(bad), off, 64));
    }
    if ((threadIdx.x & 63) == 0) {
        red_m[threadIdx.x >> 6] = m;
        red_f[threadIdx.x >> 6] = bad;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kThreads / 64; ++w) {
            m = max(m, red_m[w]);
            bad |= red_f[w];
        }
        const uint16_t h = uint16_t(m);
        const float v = DT == 1 ? float(__builtin_bit_cast(_Float16, h)) : __uint_as_float(uint32_t(h) << 16);
        // most blocks see nothing new: a (possibly stale) look at the running maximum spares the memory-side atomic
        if (__float_as_uint(v) > __builtin_nontemporal_load(&hdr->absmax_bits)) atomicMax(&hdr->absmax_bits, __float_as_uint(v));
        if (bad) atomicOr(&hdr->x_nonfinite, 1u);
    }
}

// n = count of 16-bit numbers, a multiple of 4; X 16-byte aligned.
hipError_t launch_scan_inputs16(const void* X, int dtype, uint64_t n, WsHeader* hdr, hipStream_t s)
{
    const uint64_t n2 = n / 4;
    const uint32_t blocks = uint32_t(std::min<uint64_t>((n2 / 8 + kThreads - 1) / kThreads + 1, 2048));
    if (dtype == 1)
        hipLaunchKernelGGL(scan_inputs16_kernel<1>, dim3(blocks), dim3(kThreads), 0, s, static_cast<const uint2*>(X), n2, hdr);
    else if (dtype == 2)
        hipLaunchKernelGGL(scan_inputs16_kernel<2>, dim3(blocks), dim3(kThreads), 0, s, static_cast<const uint2*>(X), n2, hdr);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

__global__ __launch_bounds__(kThreads) void zero_accumulators_kernel(long long* sums, uint32_t* counts, uint32_t K,
                                                                      uint32_t d, const uint32_t* __restrict__ gate,
                                                                      uint32_t gate_limit)
{
    if (gate != nullptr && *gate <= gate_limit) return;
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i < K * d) sums[i] = 0;
    if (i < K) counts[i] = 0;
}

template <int D>
__global__ __launch_bounds__(kThreads) void accumulate_kernel(const float* __restrict__ X, uint32_t N,
                                                              const uint32_t* __restrict__ idx, uint32_t K,
                                                              long long* sums, uint32_t* counts, WsHeader* hdr,
                                                              const uint32_t* __restrict__ gate, uint32_t gate_limit)
{
    if (gate != nullptr && *gate <= gate_limit) return;
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= N) return;
    const int e = fixed_point_exp(hdr->absmax_bits, N);
    const uint32_t k = idx[i];
    if (k >= K) {
        atomicAdd(&hdr->skipped_vectors, 1ull);
        return;
    }
    float x[D];
    load_row<D>(X + size_t(i) * D, x);
    accumulate_vector<D>(x, k, sums, counts, e, +1);
}

__global__ __launch_bounds__(kThreads) void finalize_kernel(const long long* __restrict__ sums,
                                                            const uint32_t* __restrict__ counts,
                                                            const float* prev, float* out, uint32_t* counts_out,
                                                            uint32_t K, uint32_t d, uint32_t N, WsHeader* hdr, int mean)
{
    const uint32_t t = blockIdx.x * kThreads + threadIdx.x;
    const int e = fixed_point_exp(hdr->absmax_bits, N);
    if (t == 0) hdr->fixed_point_exp = e;
    if (t >= K * d) return;
    const uint32_t k = t / d;
    const uint32_t n = counts[k];
    float c;
    if (!mean) {
        c = float(ldexp(double(sums[t]), -e));              // the plain sum (codebook gradient)
    } else if (n > 0) {
        c = float(ldexp(double(sums[t]), -e) / double(n));  // one fp64 division, one rounding to fp32
    } else {
        c = prev[t];
    }
    out[t] = c;
    if (counts_out != nullptr && t % d == 0) counts_out[k] = n;
}

hipError_t launch_zero_accumulators(const Workspace& w, uint32_t K, uint32_t d, const uint32_t* gate,
                                    uint32_t gate_limit, hipStream_t s)
{
    hipLaunchKernelGGL(zero_accumulators_kernel, dim3((K * d + kThreads - 1) / kThreads), dim3(kThreads), 0, s, w.sums,
                       w.counts, K, d, gate, gate_limit);
    return hipGetLastError();
}

hipError_t launch_accumulate(const float* X, uint32_t N, uint32_t d, const uint32_t* idx, uint32_t K,
                             const Workspace& w, const uint32_t* gate, uint32_t gate_limit, hipStream_t s)
{
    const dim3 grid((N + kThreads - 1) / kThreads);
    switch (d) {
        case 4: hipLaunchKernelGGL(accumulate_kernel<4>, grid, dim3(kThreads), 0, s, X, N, idx, K, w.sums, w.counts, w.hdr, gate, gate_limit); break;
        case 8: hipLaunchKernelGGL(accumulate_kernel<8>, grid, dim3(kThreads), 0, s, X, N, idx, K, w.sums, w.counts, w.hdr, gate, gate_limit); break;
        case 16: hipLaunchKernelGGL(accumulate_kernel<16>, grid, dim3(kThreads), 0, s, X, N, idx, K, w.sums, w.counts, w.hdr, gate, gate_limit); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_finalize(const float* prev, float* out, uint32_t* counts_out, uint32_t K, uint32_t d, uint32_t N,
                           const Workspace& w, bool mean, hipStream_t s)
{
    hipLaunchKernelGGL(finalize_kernel, dim3((K * d + kThreads - 1) / kThreads), dim3(kThreads), 0, s, w.sums, w.counts,
                       prev, out, counts_out, K, d, N, w.hdr, mean ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_update(const float* X, uint32_t N, uint32_t d, const uint32_t* idx, const float* prev, uint32_t K,
                         float* out, uint32_t* counts_out, const Workspace& w, bool mean, hipStream_t s)
{
    hipError_t e;
    if (update_sliced_applies(N, d, K, w)) {
        // many vectors: one pass over the codes per slice of the clusters, sums in LDS, the vectors are not copied
        return launch_update_sliced(X, N, d, idx, prev, K, out, counts_out, w, mean, s);
    } else if (w.bucket_ok && N >= 32768) {
        // memory-side atomics are the bottleneck of the scatter formulation: group by bucket, sum in LDS
        return launch_update_buckets(X, N, d, idx, prev, K, out, counts_out, w, false, mean, s);
    } else {
        e = launch_zero_accumulators(w, K, d, nullptr, 0, s);
        if (e != hipSuccess) return e;
        e = launch_accumulate(X, N, d, idx, K, w, nullptr, 0, s);
        if (e != hipSuccess) return e;
    }
    return launch_finalize(prev, out, counts_out, K, d, N, w, mean, s);
}

}  // namespace cc
