// Uniformly quantised codebook (the paper's inference-only variant: the codebook of a compressed layer is
// quantised to 8 or 4 bits with the symmetric uniform grid of Section 2, which shrinks it enough to speed
// up inference).
//
// Why it is faster here: a 16-bit codebook of 65536 x 4 entries (512 KB) lives in L2, and every code costs
// one L1 miss (a 128-byte line fill), which caps reconstruction and the fused forward pass at ~0.4 codes
// per clock and CU. At 4 bits the same codebook is 128 KB and fits the 160 KB of LDS of one CU: persistent
// workgroups (one per CU) copy it into LDS once and then serve every code from there, dequantising on the
// fly (q * s in fp32, rounded to the 16-bit format of the layer). Codebooks too large for LDS are read from
// global memory with the same code.
//
// Quantisation rule (one scale per codebook): s = max|c| / (2^(b-1) - 1), q = clamp(rint(c / s)), both in
// fp32; 4-bit values are two's-complement nibbles, element e in byte e/2, low nibble first.
#include <algorithm>

#include "common.h"

namespace cc {

namespace {

constexpr int kThreads = 256;

template <int DT>
__device__ __forceinline__ uint32_t to_bits16(float v)
{
    if constexpr (DT == 1) {
        return __builtin_bit_cast(uint16_t, _Float16(v));
    } else {
        const uint32_t b = __float_as_uint(v);
        if ((b & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
        return (b + 0x7fffu + ((b >> 16) & 1u)) >> 16;
    }
}

template <int DT>
__device__ __forceinline__ float from_bits16(uint16_t v)
{
    if constexpr (DT == 1) return float(__builtin_bit_cast(_Float16, v));
    else return __uint_as_float(uint32_t(v) << 16);
}

// ---- quantisation ---------------------------------------------------------------------------------
__global__ void quant_clear_kernel(uint32_t* absmax_bits)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) *absmax_bits = 0;
}

__global__ __launch_bounds__(kThreads) void quant_absmax_kernel(const float* __restrict__ c, size_t n, uint32_t* absmax_bits)
{
    uint32_t m = 0;
    for (size_t i = size_t(blockIdx.x) * kThreads + threadIdx.x; i < n; i += size_t(gridDim.x) * kThreads)
        m = max(m, __float_as_uint(c[i]) & 0x7fffffffu);
    for (int off = 32; off > 0; off >>= 1) m = max(m, uint32_t(__shfl_xor(int(m), off, 64)));
    if ((threadIdx.x & 63) == 0 && m > __builtin_nontemporal_load(absmax_bits)) atomicMax(absmax_bits, m);
}

// one thread per output byte (one element at 8 bits, two at 4 bits); thread 0 also stores the scale
template <int BITS>
__global__ __launch_bounds__(kThreads) void quantize_kernel(const float* __restrict__ c, size_t n,
                                                            const uint32_t* __restrict__ absmax_bits,
                                                            uint8_t* __restrict__ q, float* __restrict__ scale_out)
{
    constexpr int kQmax = (1 << (BITS - 1)) - 1;
    const float absmax = __uint_as_float(*absmax_bits);
    float s = absmax / float(kQmax);
    if (!(s > 0.0f) || !(s < INFINITY)) s = 0.0f;  // all-zero (or non-finite) codebook: every code is 0
    const size_t t = size_t(blockIdx.x) * kThreads + threadIdx.x;
    if (t == 0) *scale_out = s;
    auto quant = [&](size_t e) -> int {
        if (e >= n || s == 0.0f) return 0;
        const float r = __builtin_rintf(c[e] / s);  // to nearest, ties to even
        return int(fminf(fmaxf(r, float(-kQmax - 1)), float(kQmax)));
    };
    if constexpr (BITS == 8) {
        if (t < n) q[t] = uint8_t(int8_t(quant(t)));
    } else {
        if (2 * t < n) q[t] = uint8_t((quant(2 * t) & 0xF) | ((quant(2 * t + 1) & 0xF) << 4));
    }
}

// ---- dequantised row lookup: the g elements of row k as 16-bit values, two per word -------------------
template <int DT, int BITS>
__device__ __forceinline__ uint32_t dequant_pair(int q0, int q1, float s)
{
    return to_bits16<DT>(float(q0) * s) | (to_bits16<DT>(float(q1) * s) << 16);
}

__device__ __forceinline__ int nibble(uint32_t raw, int i) { return int(((raw >> (4 * i)) & 0xFu) ^ 8u) - 8; }
__device__ __forceinline__ int byte_of(uint32_t raw, int i) { return int(int8_t((raw >> (8 * i)) & 0xFFu)); }

template <int DT, int BITS>
__device__ __forceinline__ void dequant_row_words(const uint8_t* book, uint32_t k, uint32_t g, float s, uint32_t (&w)[8])
{
    if (g == 4) {
        if constexpr (BITS == 4) {
            const uint32_t raw = *reinterpret_cast<const uint16_t*>(book + 2 * size_t(k));
            w[0] = dequant_pair<DT, BITS>(nibble(raw, 0), nibble(raw, 1), s);
            w[1] = dequant_pair<DT, BITS>(nibble(raw, 2), nibble(raw, 3), s);
        } else {
            const uint32_t raw = *reinterpret_cast<const uint32_t*>(book + 4 * size_t(k));
            w[0] = dequant_pair<DT, BITS>(byte_of(raw, 0), byte_of(raw, 1), s);
            w[1] = dequant_pair<DT, BITS>(byte_of(raw, 2), byte_of(raw, 3), s);
        }
        return;
    }
    if (g == 8 && BITS == 8) {
        const uint2 raw = *reinterpret_cast<const uint2*>(book + 8 * size_t(k));
        w[0] = dequant_pair<DT, BITS>(byte_of(raw.x, 0), byte_of(raw.x, 1), s);
        w[1] = dequant_pair<DT, BITS>(byte_of(raw.x, 2), byte_of(raw.x, 3), s);
        w[2] = dequant_pair<DT, BITS>(byte_of(raw.y, 0), byte_of(raw.y, 1), s);
        w[3] = dequant_pair<DT, BITS>(byte_of(raw.y, 2), byte_of(raw.y, 3), s);
        return;
    }
    if (g == 8 && BITS == 4) {
        const uint32_t raw = *reinterpret_cast<const uint32_t*>(book + 4 * size_t(k));
#pragma unroll
        for (int q = 0; q < 4; ++q) w[q] = dequant_pair<DT, BITS>(nibble(raw, 2 * q), nibble(raw, 2 * q + 1), s);
        return;
    }
    const size_t e0 = size_t(k) * g;
#pragma unroll
    for (uint32_t q = 0; q < 8; ++q) {
        if (2 * q >= g) break;
        int v[2] = {0, 0};
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const size_t e = e0 + 2 * q + i;
            if (2 * q + i >= g) continue;
            if constexpr (BITS == 4) v[i] = nibble(book[e >> 1], int(e & 1));
            else v[i] = int(int8_t(book[e]));
        }
        w[q] = dequant_pair<DT, BITS>(v[0], v[1], s);
    }
}

// Copies the codebook into LDS: whole 16-byte pieces, then the last few bytes one by one. Every workgroup of
// the grid copies the same bytes at the same time, so each starts at a different place: in step they would
// all queue on one L2 channel after the other.
__device__ __forceinline__ void stage_book(const uint8_t* __restrict__ src, uint32_t bytes, uint8_t* dst)
{
    const uint32_t pieces = bytes / 16;
    const uint32_t rot = pieces ? uint32_t((uint64_t(blockIdx.x) * 2654435761ull) % pieces) : 0u;
    constexpr int U = 16;  // loads in flight per thread: with few waves per CU the copy is latency-bound
    for (uint32_t i0 = threadIdx.x; i0 < pieces; i0 += blockDim.x * U) {
        uint4 t[U];
        uint32_t at[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t i = i0 + u * blockDim.x;
            at[u] = i < pieces ? (i + rot >= pieces ? i + rot - pieces : i + rot) : 0xffffffffu;
            t[u] = *reinterpret_cast<const uint4*>(src + size_t(at[u] == 0xffffffffu ? 0u : at[u]) * 16);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (at[u] != 0xffffffffu) *reinterpret_cast<uint4*>(dst + size_t(at[u]) * 16) = t[u];
    }
    for (uint32_t o = pieces * 16 + threadIdx.x; o < bytes; o += blockDim.x) dst[o] = src[o];
    __syncthreads();
}

// ---- reconstruction --------------------------------------------------------------------------------
// Persistent workgroups stride over the codes; one lane per code writes its g elements (padding cut).
template <int DT, int BITS, bool IN_LDS>
__global__ __launch_bounds__(1024) void layer_weight_q_kernel(const uint8_t* __restrict__ qbook, uint32_t book_bytes,
                                                               const float* __restrict__ scale, uint32_t K, uint32_t g,
                                                               const uint16_t* __restrict__ codes, uint64_t num_codes,
                                                               uint32_t per_row, uint32_t out_features,
                                                               uint16_t* __restrict__ weight)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const uint8_t* book = qbook;
    if constexpr (IN_LDS) {
        stage_book(qbook, book_bytes, smem);
        book = smem;
    }
    const float s = *scale;
    const bool whole4 = g == 4 && out_features % 4 == 0;
    const bool whole8 = g == 8 && out_features % 8 == 0;
    constexpr int U = 8;  // codes in flight per lane: one code per step would leave the loop latency-bound
    const uint64_t stride = uint64_t(gridDim.x) * blockDim.x;
    for (uint64_t v0 = uint64_t(blockIdx.x) * blockDim.x + threadIdx.x; v0 < num_codes; v0 += stride * U) {
        uint32_t ks[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t v = v0 + u * stride;
            ks[u] = v < num_codes ? min(uint32_t(codes[v]), K - 1) : 0u;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint64_t v = v0 + u * stride;
            if (v >= num_codes) break;
            uint32_t w[8];
            dequant_row_words<DT, BITS>(book, ks[u], g, s, w);
            if (whole4) {
                typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                __builtin_nontemporal_store(u32x2{w[0], w[1]}, reinterpret_cast<u32x2*>(weight) + v);
            } else if (whole8) {
                typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
                __builtin_nontemporal_store(u32x4{w[0], w[1], w[2], w[3]}, reinterpret_cast<u32x4*>(weight) + v);
            } else {
                const uint32_t r = uint32_t(v / per_row), c = uint32_t(v % per_row) * g;
                uint16_t* dst = weight + size_t(r) * out_features + c;
                const uint32_t n = min(g, out_features - c);
#pragma unroll
                for (uint32_t j = 0; j < 16; ++j)
                    if (j < n) dst[j] = uint16_t(w[j >> 1] >> (16 * (j & 1)));
            }
        }
    }
}

// ---- fused forward ---------------------------------------------------------------------------------
constexpr int BN = 64, BK = 64, S = BK / 2 + 4;
constexpr uint32_t kTileBytes = BN * S * 4;  // Wt; the 8 KB reduction buffer aliases it

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int DT>
__device__ __forceinline__ f32x16 mma(u32x4 a, u32x4 b, f32x16 c)
{
    if constexpr (DT == 1)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// Same tiling as the 16-bit forward kernel (32*MT rows x 64 columns x a slice of in-features per job, 4 waves
// each owning a 16-wide k slice of every 64-wide step), but the workgroups are persistent: each copies the
// codebook into LDS once and then walks its jobs. It serves g other than 4 and 8, M above 16, and codebooks too
// large for LDS (then read from global memory by four workgroups per CU); decode-time shapes take the few-rows
// kernel below.
template <int DT, int MT, int BITS, bool IN_LDS>
__global__ __launch_bounds__(kThreads) void layer_forward_q_kernel(
    const uint16_t* __restrict__ x, uint32_t M, const uint8_t* __restrict__ qbook, uint32_t book_bytes,
    const float* __restrict__ scale, uint32_t K, uint32_t g, const uint16_t* __restrict__ codes, uint32_t per_row,
    uint32_t in_features, uint32_t out_features, const uint16_t* __restrict__ bias, uint16_t* __restrict__ y,
    float* __restrict__ partial, uint32_t n_tiles, uint32_t splits, uint32_t rows_per_split, uint32_t m_tiles)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    uint32_t* Wt = reinterpret_cast<uint32_t*>(smem);
    float (*red)[16][64] = reinterpret_cast<float (*)[16][64]>(smem);  // [2][16][64], used between k loops only
    const uint8_t* book = qbook;
    if constexpr (IN_LDS) {
        stage_book(qbook, book_bytes, smem + kTileBytes);
        book = smem + kTileBytes;
    }
    const float s = *scale;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, h = lane >> 5;
    const uint32_t jobs = n_tiles * splits * m_tiles;

    // geometry of a job
    struct Job { uint32_t n_lo, m0, split, k_begin, k_end, cn_lo, cpr, items; };
    auto job_of = [&](uint32_t j) {
        Job q;
        const uint32_t nt = j % n_tiles, rest = j / n_tiles;  // neighbouring workgroups: neighbouring column tiles
        q.split = rest % splits;
        q.m0 = (rest / splits) * (32 * MT);
        q.n_lo = nt * BN;
        q.k_begin = q.split * rows_per_split;
        q.k_end = min(q.k_begin + rows_per_split, in_features);
        q.cn_lo = q.n_lo / g;
        const uint32_t cn_hi = min((q.n_lo + BN - 1) / g, per_row - 1);
        q.cpr = cn_hi - q.cn_lo + 1;
        q.items = (BK / 2) * q.cpr;
        return q;
    };
    uint32_t j = blockIdx.x;
    if (j >= jobs) return;
    Job q = job_of(j);

    while (true) {
        f32x16 acc[MT][2];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mt][nb][r] = 0.0f;

        const uint32_t jn = j + gridDim.x;
        const bool more_jobs = jn < jobs;
        const Job qn = more_jobs ? job_of(jn) : q;

        for (uint32_t k0 = q.k_begin; k0 < q.k_end; k0 += BK) {
            // this lane's A operands
            const uint32_t kk = k0 + 16 * wave + 8 * h;
            u32x4 a[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const uint32_t m = q.m0 + 32 * mt + (lane & 31);
                a[mt] = u32x4{0u, 0u, 0u, 0u};
                if (m < M && kk < q.k_end) a[mt] = *reinterpret_cast<const u32x4*>(x + size_t(m) * in_features + kk);
            }
            // gather the W piece from the codebook: Wt[n - n_lo][k - k0], two k per word
            for (uint32_t it = threadIdx.x; it < q.items; it += kThreads) {
                const uint32_t rp = it / q.cpr, c = it % q.cpr;
                const uint32_t r0 = k0 + 2 * rp, r1 = r0 + 1;
                const bool live0 = r0 < q.k_end, live1 = r1 < q.k_end;
                const uint32_t code0 = live0 ? min(uint32_t(codes[size_t(r0) * per_row + q.cn_lo + c]), K - 1) : 0u;
                const uint32_t code1 = live1 ? min(uint32_t(codes[size_t(r1) * per_row + q.cn_lo + c]), K - 1) : 0u;
                uint32_t w0[8], w1[8];
                // the B operand holds the integers q themselves (exact in either 16-bit format); the scale is
                // applied once to the finished sum
                dequant_row_words<DT, BITS>(book, code0, g, 1.0f, w0);
                dequant_row_words<DT, BITS>(book, code1, g, 1.0f, w1);
                const int nbase = int((q.cn_lo + c) * g) - int(q.n_lo);
#pragma unroll
                for (uint32_t e = 0; e < 16; ++e) {
                    if (e >= g) break;
                    const int n = nbase + int(e);
                    if (n < 0 || n >= BN) continue;
                    const uint32_t e0 = live0 ? (w0[e >> 1] >> (16 * (e & 1))) & 0xffffu : 0u;
                    const uint32_t e1 = live1 ? (w1[e >> 1] >> (16 * (e & 1))) & 0xffffu : 0u;
                    Wt[n * S + rp] = e0 | (e1 << 16);
                }
            }
            __syncthreads();
            u32x4 b[2];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
                b[nb] = *reinterpret_cast<const u32x4*>(&Wt[(32 * nb + (lane & 31)) * S + 8 * wave + 4 * h]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb) acc[mt][nb] = mma<DT>(a[mt], b[nb], acc[mt][nb]);
            __syncthreads();
        }

        // add the four k slices: (w0 + w2) + (w1 + w3), through the 8 KB buffer that aliases Wt; wave 0 stores
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                if (wave >= 2) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) red[wave - 2][r][lane] = acc[mt][nb][r];
                }
                __syncthreads();
                if (wave < 2) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[mt][nb][r] += red[wave][r][lane];
                }
                __syncthreads();
                if (wave == 1) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) red[0][r][lane] = acc[mt][nb][r];
                }
                __syncthreads();
                if (wave == 0) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float v = (acc[mt][nb][r] + red[0][r][lane]) * (splits == 1 ? s : 1.0f);
                        const uint32_t m = q.m0 + 32 * mt + (r & 3) + 8 * (r >> 2) + 4 * h;
                        const uint32_t n = q.n_lo + 32 * nb + (lane & 31);
                        if (m < M && n < out_features) {
                            if (splits == 1) {
                                y[size_t(m) * out_features + n] =
                                    uint16_t(to_bits16<DT>(bias ? v + from_bits16<DT>(bias[n]) : v));
                            } else {
                                partial[(size_t(q.split) * M + m) * out_features + n] = v;
                            }
                        }
                    }
                }
                __syncthreads();
            }
        }
        if (!more_jobs) break;
        j = jn;
        q = qn;
    }
}

// Row k of the quantised codebook as floats with the offset left in: f[j] = q[j] + 2^(BITS-1), an unsigned byte
// that converts to float in one instruction (the offset is removed once per wave, see the kernel).
template <int BITS, int G>
__device__ __forceinline__ void biased_row(const uint8_t* book, uint32_t k, float (&f)[G])
{
    uint32_t packed[G / 4];  // byte i of word v: element order given by `lane_of`
    if constexpr (BITS == 8) {
#pragma unroll
        for (int v = 0; v < G / 4; ++v)
            packed[v] = reinterpret_cast<const uint32_t*>(book + size_t(k) * G)[v] ^ 0x80808080u;
#pragma unroll
        for (int j = 0; j < G; ++j) f[j] = float((packed[j / 4] >> (8 * (j % 4))) & 0xffu);
    } else {
        // 4 nibbles n3 n2 n1 n0 -> bytes (n0, n2, n1, n3), each xor 8
#pragma unroll
        for (int v = 0; v < G / 4; ++v) {
            const uint32_t r = reinterpret_cast<const uint16_t*>(book + size_t(k) * (G / 2))[v];
            packed[v] = ((r & 0x0f0fu) | (((r >> 4) & 0x0f0fu) << 16)) ^ 0x08080808u;
        }
#pragma unroll
        for (int j = 0; j < G; ++j) {
            const int e = j % 4;
            const int byte = e == 0 ? 0 : (e == 1 ? 2 : (e == 2 ? 1 : 3));
            f[j] = float((packed[j / 4] >> (8 * byte)) & 0xffu);
        }
    }
}

// ---- fused forward on the matrix cores with the codebook in LDS, g = 4 or 8, up to 64 rows of x ---------------
// The tiling of the kernel above with everything the compiler needs to know at compile time: with g fixed, a
// step of 64 in-features x 64 columns is exactly NI items (two codebook rows each) per thread, so the codes and
// the x operands of the next step sit in a fixed number of registers while the current step is gathered from
// LDS, written to the transposed tile and multiplied. B holds the integers q (exact in bf16 and fp16).
// Measured: 43 us for a 4096 x 4096 layer whatever M <= 32 (58 us for M <= 64): the four waves of the one
// workgroup a CU can hold spend most of their time waiting (a three-step-deep operand ring did not help), so
// this kernel only takes over where the few-rows kernel's M * g multiply-adds per code cost more (M > 16).
template <int BITS, int G>
__device__ __forceinline__ void signed_row(const uint8_t* book, uint32_t k, float (&f)[G])
{
    biased_row<BITS, G>(book, k, f);
#pragma unroll
    for (int j = 0; j < G; ++j) f[j] -= float(1 << (BITS - 1));
}

template <int DT, int BITS, int G, int MT>
__global__ __launch_bounds__(kThreads) void layer_forward_q_mfma_kernel(
    const uint16_t* __restrict__ x, uint32_t M, const uint8_t* __restrict__ qbook, uint32_t book_bytes,
    const float* __restrict__ scale, uint32_t K, const uint16_t* __restrict__ codes, uint32_t per_row,
    uint32_t in_features, uint32_t out_features, const uint16_t* __restrict__ bias, uint16_t* __restrict__ y,
    float* __restrict__ partial, uint32_t n_tiles, uint32_t splits, uint32_t rows_per_split)
{
    constexpr int CPR = BN / G;                        // code columns of a tile
    constexpr int NI = (BK / 2) * CPR / kThreads;      // items per thread and step
    static_assert((BK / 2) * CPR % kThreads == 0, "whole items per thread");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    uint32_t* Wt = reinterpret_cast<uint32_t*>(smem);
    float (*red)[16][64] = reinterpret_cast<float (*)[16][64]>(smem);  // [2][16][64], used between k loops only
    uint8_t* book = smem + kTileBytes;
    stage_book(qbook, book_bytes, book);
    const float s = *scale;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, h = lane >> 5;
    const uint32_t jobs = n_tiles * splits;

    // item i of this thread: row pair rp[i] of the step, code column cc[i] of the tile
    uint32_t rp[NI], cc[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const uint32_t it = threadIdx.x + i * kThreads;
        rp[i] = it / CPR;
        cc[i] = it % CPR;
    }
    auto fetch_codes = [&](uint32_t n_lo, uint32_t k0, uint32_t k_end, uint32_t (&pc)[NI]) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const uint32_t cn = n_lo / G + cc[i];
            const uint32_t r0 = k0 + 2 * rp[i];
            const bool on = cn < per_row && r0 < k_end;  // k_end is even: the pair is in or out as a whole
            const uint32_t c0 = on ? codes[size_t(r0) * per_row + cn] : 0u;
            const uint32_t c1 = on ? codes[size_t(r0 + 1) * per_row + cn] : 0u;
            pc[i] = c0 | (c1 << 16) | 0u;
        }
    };
    auto fetch_x = [&](uint32_t k0, uint32_t k_end, u32x4 (&a)[MT]) {
        const uint32_t kk = k0 + 16 * wave + 8 * h;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const uint32_t m = 32 * mt + (lane & 31);
            a[mt] = u32x4{0u, 0u, 0u, 0u};
            if (m < M && kk < k_end) a[mt] = *reinterpret_cast<const u32x4*>(x + size_t(m) * in_features + kk);
        }
    };
    auto span = [&](uint32_t job, uint32_t& n_lo, uint32_t& split, uint32_t& k_begin, uint32_t& k_end) {
        n_lo = (job % n_tiles) * BN;
        split = job / n_tiles;
        k_begin = split * rows_per_split;
        k_end = min(k_begin + rows_per_split, in_features);
    };

    uint32_t job = blockIdx.x;
    if (job >= jobs) return;
    uint32_t n_lo, split, k_begin, k_end;
    span(job, n_lo, split, k_begin, k_end);
    uint32_t pc[NI];
    u32x4 a[MT];
    fetch_codes(n_lo, k_begin, k_end, pc);
    fetch_x(k_begin, k_end, a);

    while (true) {
        f32x16 acc[MT][2];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mt][nb][r] = 0.0f;
        const uint32_t next_job = job + gridDim.x;
        const bool more = next_job < jobs;
        uint32_t nn_lo = n_lo, nsplit = split, nk_begin = k_begin, nk_end = k_end;
        if (more) span(next_job, nn_lo, nsplit, nk_begin, nk_end);

        for (uint32_t k0 = k_begin; k0 < k_end; k0 += BK) {
            // request the operands of the step after this one (same job, or the first step of the next job)
            uint32_t nc[NI];
            u32x4 na[MT];
            const bool last = k0 + BK >= k_end;
            if (!last) {
                fetch_codes(n_lo, k0 + BK, k_end, nc);
                fetch_x(k0 + BK, k_end, na);
            } else {
                fetch_codes(nn_lo, nk_begin, more ? nk_end : 0u, nc);
                fetch_x(nk_begin, more ? nk_end : 0u, na);
            }
            // gather this step's piece of W from LDS into the transposed tile
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const uint32_t cn = n_lo / G + cc[i];
                const bool on = cn < per_row && k0 + 2 * rp[i] < k_end;
                float f0[G], f1[G];
                signed_row<BITS, G>(book, min(pc[i] & 0xffffu, K - 1), f0);
                signed_row<BITS, G>(book, min(pc[i] >> 16, K - 1), f1);
#pragma unroll
                for (int e = 0; e < G; ++e) {
                    const uint32_t lo16 = on ? to_bits16<DT>(f0[e]) : 0u, hi16 = on ? to_bits16<DT>(f1[e]) : 0u;
                    Wt[(cc[i] * G + e) * S + rp[i]] = lo16 | (hi16 << 16);
                }
            }
            __syncthreads();
            u32x4 b[2];
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
                b[nb] = *reinterpret_cast<const u32x4*>(&Wt[(32 * nb + (lane & 31)) * S + 8 * wave + 4 * h]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nb = 0; nb < 2; ++nb) acc[mt][nb] = mma<DT>(a[mt], b[nb], acc[mt][nb]);
            __syncthreads();
#pragma unroll
            for (int i = 0; i < NI; ++i) pc[i] = nc[i];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) a[mt] = na[mt];
        }

        // add the four k slices: (w0 + w2) + (w1 + w3), through the 8 KB buffer that aliases the tile; wave 0 stores
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                if (wave >= 2) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) red[wave - 2][r][lane] = acc[mt][nb][r];
                }
                __syncthreads();
                if (wave < 2) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[mt][nb][r] += red[wave][r][lane];
                }
                __syncthreads();
                if (wave == 1) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) red[0][r][lane] = acc[mt][nb][r];
                }
                __syncthreads();
                if (wave == 0) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float v = (acc[mt][nb][r] + red[0][r][lane]) * (splits == 1 ? s : 1.0f);
                        const uint32_t m = 32 * mt + (r & 3) + 8 * (r >> 2) + 4 * h;
                        const uint32_t n = n_lo + 32 * nb + (lane & 31);
                        if (m < M && n < out_features) {
                            if (splits == 1) {
                                y[size_t(m) * out_features + n] =
                                    uint16_t(to_bits16<DT>(bias ? v + from_bits16<DT>(bias[n]) : v));
                            } else {
                                partial[(size_t(split) * M + m) * out_features + n] = v;
                            }
                        }
                    }
                }
                __syncthreads();
            }
        }
        if (!more) break;
        job = next_job;
        n_lo = nn_lo; split = nsplit; k_begin = nk_begin; k_end = nk_end;
    }
}

// ---- fused forward for few rows of x (decode-time M <= 16), codebook in LDS, g = 4 or 8 ------------------
// No matrix cores and no transposition: a lane owns one code column (g outputs) and walks down the
// in-features of its slice; per code it looks the row up in LDS, dequantises it, and does MB * g fused
// multiply-adds against x values that are uniform over the wave (scalar loads). 8 waves of a workgroup share
// 64 code columns and take every 8th pair of in-features; their partial sums meet in LDS at the end.
// The sum runs over x * q with the integers q (exact products); the scale multiplies the finished sum.
constexpr int kGemvThreads = 512, kGemvWaves = 8, kGemvCols = 64;


template <int DT, int BITS, int G, int MB>
__global__ __launch_bounds__(kGemvThreads) void layer_forward_q_gemv_kernel(
    const uint16_t* __restrict__ x, uint32_t M, const uint8_t* __restrict__ qbook, uint32_t book_bytes,
    const float* __restrict__ scale, uint32_t K, const uint16_t* __restrict__ codes, uint32_t per_row,
    uint32_t in_features, uint32_t out_features, const uint16_t* __restrict__ bias, uint16_t* __restrict__ y,
    float* __restrict__ partial, uint32_t col_blocks, uint32_t splits, uint32_t rows_per_split)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    constexpr int MC = G == 4 ? 2 : 1;                           // rows of x per reduction round (16 KB of LDS)
    float* red = reinterpret_cast<float*>(smem);                 // [kGemvWaves][MC][kGemvCols * G]
    constexpr uint32_t kRedBytes = kGemvWaves * MC * kGemvCols * G * 4;
    uint8_t* book = smem + kRedBytes;
    stage_book(qbook, book_bytes, book);
    const float s = *scale;
    const int lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t jobs = col_blocks * splits;

    for (uint32_t job = blockIdx.x; job < jobs; job += gridDim.x) {
        const uint32_t cb = job % col_blocks, split = job / col_blocks;
        const uint32_t cn = cb * kGemvCols + lane;
        const bool live = cn < per_row;
        const uint32_t k_begin = split * rows_per_split, k_end = min(k_begin + rows_per_split, in_features);
        float acc[MB][G], xsum[MB];
#pragma unroll
        for (int m = 0; m < MB; ++m) {
            xsum[m] = 0.0f;
#pragma unroll
            for (int j = 0; j < G; ++j) acc[m][j] = 0.0f;
        }

        // pairs of in-features (rows 2p, 2p + 1): this wave takes p = k_begin/2 + wave, + 8, ...; the codes of
        // U pairs are requested before any is used
        constexpr int U = MB >= 16 ? 4 : 8;
        uint32_t c0[U], c1[U];
        auto fetch = [&](uint32_t p0, uint32_t (&a0)[U], uint32_t (&a1)[U]) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t p = p0 + u * kGemvWaves;
                const bool on = live && 2 * p < k_end;
                a0[u] = on ? uint32_t(codes[size_t(2 * p) * per_row + cn]) : 0u;
                a1[u] = on ? uint32_t(codes[size_t(2 * p + 1) * per_row + cn]) : 0u;
            }
        };
        uint32_t p0 = k_begin / 2 + wave;
        fetch(p0, c0, c1);
        for (; 2 * p0 < k_end; p0 += kGemvWaves * U) {
            // the next batch is requested before this one is used: its latency hides behind the arithmetic
            uint32_t n0[U], n1[U];
            fetch(p0 + kGemvWaves * U, n0, n1);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t p = p0 + u * kGemvWaves;
                if (2 * p >= k_end) break;  // wave-uniform
                float f0[G], f1[G];
                biased_row<BITS, G>(book, min(c0[u], K - 1), f0);
                biased_row<BITS, G>(book, min(c1[u], K - 1), f1);
#pragma unroll
                for (int m = 0; m < MB; ++m) {
                    // both x values of the pair in one (wave-uniform) 32-bit load
                    const uint32_t xw = m < int(M) ? reinterpret_cast<const uint32_t*>(x + size_t(m) * in_features)[p] : 0u;
                    const float x0 = from_bits16<DT>(uint16_t(xw & 0xffffu)), x1 = from_bits16<DT>(uint16_t(xw >> 16));
                    xsum[m] += x0 + x1;
#pragma unroll
                    for (int j = 0; j < G; ++j) {
                        acc[m][j] = __builtin_fmaf(x0, f0[j], acc[m][j]);
                        acc[m][j] = __builtin_fmaf(x1, f1[j], acc[m][j]);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                c0[u] = n0[u];
                c1[u] = n1[u];
            }
        }
        // the stored integers were taken with their offset (q + 2^(BITS-1)): remove offset * sum of this wave's x
#pragma unroll
        for (int m = 0; m < MB; ++m)
#pragma unroll
            for (int j = 0; j < G; ++j) acc[m][j] = __builtin_fmaf(-float(1 << (BITS - 1)), xsum[m], acc[m][j]);

        // sum over the 8 waves, MC rows of x per round: thread t finishes element t of the round
#pragma unroll
        for (int m0 = 0; m0 < MB; m0 += MC) {
            __syncthreads();
#pragma unroll
            for (int mc = 0; mc < MC; ++mc)
#pragma unroll
                for (int j = 0; j < G; ++j)
                    if (m0 + mc < MB) red[((wave * MC + mc) * kGemvCols + lane) * G + j] = acc[(m0 + mc) % MB][j];
            __syncthreads();
            constexpr int kRound = MC * kGemvCols * G;  // elements per round
            for (int t = threadIdx.x; t < kRound; t += kGemvThreads) {
                const int mc = t / (kGemvCols * G), rest = t % (kGemvCols * G);
                float v = 0.0f;
#pragma unroll
                for (int w = 0; w < kGemvWaves; ++w) v += red[(w * MC + mc) * kGemvCols * G + rest];
                if (splits == 1) v *= s;
                const uint32_t m = m0 + mc;
                const uint32_t n = cb * kGemvCols * G + rest;
                if (m < M && m < MB && n < out_features) {
                    if (splits == 1) {
                        y[size_t(m) * out_features + n] = uint16_t(to_bits16<DT>(bias ? v + from_bits16<DT>(bias[n]) : v));
                    } else {
                        partial[(size_t(split) * M + m) * out_features + n] = v;
                    }
                }
            }
        }
        __syncthreads();
    }
}

template <int DT>
__global__ __launch_bounds__(kThreads) void forward_q_reduce_kernel(const float* __restrict__ partial, uint64_t n,
                                                                    uint32_t out_features, uint32_t splits,
                                                                    const float* __restrict__ scale,
                                                                    const uint16_t* __restrict__ bias,
                                                                    uint16_t* __restrict__ y)
{
    const uint64_t t = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
    if (t >= n) return;
    float v = partial[t];
    for (uint32_t s = 1; s < splits; ++s) v += partial[uint64_t(s) * n + t];  // fixed order
    v *= *scale;
    if (bias) v += from_bits16<DT>(bias[t % out_features]);
    y[t] = uint16_t(to_bits16<DT>(v));
}

int g_cus = 0;
int compute_units()
{
    if (g_cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        g_cus = n;
    }
    return g_cus;
}

// Kernels that keep the codebook in LDS need more than the default 64 KB of dynamic LDS.
template <typename Kernel>
hipError_t allow_lds(Kernel kernel, uint32_t bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, int(bytes));
}

}  // namespace

// Largest codebook (bytes) that the persistent kernels keep in LDS next to their tile buffers.
constexpr uint32_t kMaxLdsBook = 128 * 1024;

hipError_t launch_codebook_quantize(const float* centroids, size_t n, int bits, void* qbook, float* scale,
                                    uint32_t* absmax_scratch, hipStream_t s)
{
    hipLaunchKernelGGL(quant_clear_kernel, dim3(1), dim3(64), 0, s, absmax_scratch);
    hipLaunchKernelGGL(quant_absmax_kernel, dim3(uint32_t(std::min<size_t>((n + kThreads - 1) / kThreads, 256))),
                       dim3(kThreads), 0, s, centroids, n, absmax_scratch);
    uint8_t* q = static_cast<uint8_t*>(qbook);
    if (bits == 8) {
        hipLaunchKernelGGL(quantize_kernel<8>, dim3(uint32_t((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, centroids, n,
                           absmax_scratch, q, scale);
    } else if (bits == 4) {
        const size_t nb = (n + 1) / 2;
        hipLaunchKernelGGL(quantize_kernel<4>, dim3(uint32_t((nb + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, centroids, n,
                           absmax_scratch, q, scale);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int DT, int BITS>
static hipError_t weight_q_t(const uint8_t* qbook, uint32_t book_bytes, const float* scale, uint32_t K, uint32_t g,
                             const uint16_t* codes, uint64_t num_codes, uint32_t per_row, uint32_t out_features,
                             uint16_t* weight, hipStream_t s)
{
    const uint32_t padded = (book_bytes + 15) & ~15u;
    const dim3 grid(uint32_t(std::min<uint64_t>(uint64_t(compute_units()), (num_codes + 1023) / 1024)));
    if (padded <= kMaxLdsBook) {
        auto kernel = layer_weight_q_kernel<DT, BITS, true>;
        hipError_t e = allow_lds(kernel, padded);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kernel, grid, dim3(1024), padded, s, qbook, book_bytes, scale, K, g, codes, num_codes, per_row,
                           out_features, weight);
    } else {
        const dim3 wide(uint32_t(std::min<uint64_t>(uint64_t(compute_units()) * 2, (num_codes + 1023) / 1024)));
        hipLaunchKernelGGL((layer_weight_q_kernel<DT, BITS, false>), wide, dim3(1024), 0, s, qbook, book_bytes, scale, K, g, codes,
                           num_codes, per_row, out_features, weight);
    }
    return hipGetLastError();
}

hipError_t launch_layer_weight_q(const void* qbook, int bits, const float* scale, uint32_t K, uint32_t g,
                                 const uint16_t* codes, uint32_t in_features, uint32_t out_features, int dtype, void* weight,
                                 hipStream_t s)
{
    const uint32_t per_row = (out_features + g - 1) / g;
    const uint64_t num_codes = uint64_t(in_features) * per_row;
    const uint32_t book_bytes = uint32_t((uint64_t(K) * g * bits + 7) / 8);
    const uint8_t* qb = static_cast<const uint8_t*>(qbook);
    uint16_t* w = static_cast<uint16_t*>(weight);
    if (dtype == 1 && bits == 4) return weight_q_t<1, 4>(qb, book_bytes, scale, K, g, codes, num_codes, per_row, out_features, w, s);
    if (dtype == 1 && bits == 8) return weight_q_t<1, 8>(qb, book_bytes, scale, K, g, codes, num_codes, per_row, out_features, w, s);
    if (dtype == 2 && bits == 4) return weight_q_t<2, 4>(qb, book_bytes, scale, K, g, codes, num_codes, per_row, out_features, w, s);
    if (dtype == 2 && bits == 8) return weight_q_t<2, 8>(qb, book_bytes, scale, K, g, codes, num_codes, per_row, out_features, w, s);
    return hipErrorInvalidValue;
}

// The few-rows kernel: 64 code columns per job; slices of in_features so that every CU gets a job or two.
static uint32_t gemv_splits(uint32_t in_features, uint32_t per_row)
{
    const uint32_t col_blocks = (per_row + kGemvCols - 1) / kGemvCols;
    uint32_t splits = (2 * 256 + col_blocks - 1) / col_blocks;
    splits = std::min<uint32_t>(splits, std::max<uint32_t>(1, in_features / (2 * kGemvWaves * 4)));  // >= 4 pairs per wave
    return std::max<uint32_t>(1, std::min<uint32_t>(splits, 64));
}

template <int DT, int BITS, int G, int MB>
static hipError_t forward_q_gemv_t(const uint16_t* x, uint32_t M, const uint8_t* qbook, uint32_t book_bytes,
                                   const float* scale, uint32_t K, const uint16_t* codes, uint32_t in_features,
                                   uint32_t out_features, const uint16_t* bias, uint16_t* y, float* partial, hipStream_t s)
{
    const uint32_t per_row = (out_features + G - 1) / G;
    const uint32_t col_blocks = (per_row + kGemvCols - 1) / kGemvCols;
    const uint32_t req = gemv_splits(in_features, per_row);
    // slices hold whole groups of 16 in-features (one pair per wave), so that every slice starts at wave 0's pair
    const uint32_t groups = (in_features + 2 * kGemvWaves - 1) / (2 * kGemvWaves);
    const uint32_t rows_per_split = (groups + req - 1) / req * (2 * kGemvWaves);
    const uint32_t splits = (in_features + rows_per_split - 1) / rows_per_split;
    auto kernel = layer_forward_q_gemv_kernel<DT, BITS, G, MB>;
    const uint32_t lds = kGemvWaves * (G == 4 ? 2 : 1) * kGemvCols * G * 4 + ((book_bytes + 15) & ~15u);
    hipError_t e = allow_lds(kernel, lds);
    if (e != hipSuccess) return e;
    const dim3 grid(std::min<uint32_t>(uint32_t(compute_units()), col_blocks * splits));
    hipLaunchKernelGGL(kernel, grid, dim3(kGemvThreads), lds, s, x, M, qbook, book_bytes, scale, K, codes, per_row, in_features,
                       out_features, bias, y, partial, col_blocks, splits, rows_per_split);
    if (splits > 1) {
        const uint64_t n = uint64_t(M) * out_features;
        hipLaunchKernelGGL(forward_q_reduce_kernel<DT>, dim3(uint32_t((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, s,
                           partial, n, out_features, splits, scale, bias, y);
    }
    return hipGetLastError();
}

static bool lds_book_applies(uint32_t K, uint32_t g, int bits)
{
    return (g == 4 || g == 8) && (uint64_t(K) * g * bits + 7) / 8 <= kMaxLdsBook;
}

template <int DT, int BITS, int G, int MT>
static hipError_t forward_q_mfma_t(const uint16_t* x, uint32_t M, const uint8_t* qbook, uint32_t book_bytes,
                                   const float* scale, uint32_t K, const uint16_t* codes, uint32_t in_features,
                                   uint32_t out_features, const uint16_t* bias, uint16_t* y, float* partial, hipStream_t s)
{
    const uint32_t per_row = (out_features + G - 1) / G;
    const uint32_t n_tiles = (out_features + BN - 1) / BN;
    const uint32_t ksteps = (in_features + BK - 1) / BK;
    uint32_t req = (2 * 256 + n_tiles - 1) / n_tiles;
    req = std::max<uint32_t>(1, std::min<uint32_t>(std::min<uint32_t>(req, 64), std::max<uint32_t>(1, ksteps / 4)));
    const uint32_t rows_per_split = (ksteps + req - 1) / req * BK;
    const uint32_t splits = (in_features + rows_per_split - 1) / rows_per_split;
    auto kernel = layer_forward_q_mfma_kernel<DT, BITS, G, MT>;
    const uint32_t lds = kTileBytes + ((book_bytes + 15) & ~15u);
    hipError_t e = allow_lds(kernel, lds);
    if (e != hipSuccess) return e;
    const dim3 grid(std::min<uint32_t>(uint32_t(compute_units()), n_tiles * splits));
    hipLaunchKernelGGL(kernel, grid, dim3(kThreads), lds, s, x, M, qbook, book_bytes, scale, K, codes, per_row, in_features,
                       out_features, bias, y, partial, n_tiles, splits, rows_per_split);
    if (splits > 1) {
        const uint64_t n = uint64_t(M) * out_features;
        hipLaunchKernelGGL(forward_q_reduce_kernel<DT>, dim3(uint32_t((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, s,
                           partial, n, out_features, splits, scale, bias, y);
    }
    return hipGetLastError();
}

// Slices of in_features per column tile: enough jobs for two rounds over the chip.
uint32_t layer_forward_q_splits(uint64_t M, uint32_t in_features, uint32_t out_features)
{
    const uint64_t n_tiles = (out_features + BN - 1) / BN;
    const int mt = M > 64 ? 4 : (M > 32 ? 2 : 1);
    const uint64_t m_tiles = (M + 32 * mt - 1) / (32 * mt);
    const uint64_t ksteps = (in_features + BK - 1) / BK;
    uint64_t splits = (2 * 256 + n_tiles * m_tiles - 1) / (n_tiles * m_tiles);
    splits = std::min<uint64_t>(splits, std::max<uint64_t>(1, ksteps / 4));  // at least four steps per slice
    return uint32_t(std::max<uint64_t>(1, std::min<uint64_t>(splits, 64)));
}

// Upper bound over both kernels (the few-rows kernel may use up to 64 slices): sizes the partial buffer.
uint32_t layer_forward_q_max_splits(uint64_t M, uint32_t in_features, uint32_t out_features)
{
    return M <= 64 ? 64u : layer_forward_q_splits(M, in_features, out_features);
}

template <int DT, int MT, int BITS>
static hipError_t forward_q_t(const uint16_t* x, uint32_t M, const uint8_t* qbook, uint32_t book_bytes, const float* scale,
                              uint32_t K, uint32_t g, const uint16_t* codes, uint32_t in_features, uint32_t out_features,
                              const uint16_t* bias, uint16_t* y, float* partial, hipStream_t s)
{
    const uint32_t per_row = (out_features + g - 1) / g;
    const uint32_t n_tiles = (out_features + BN - 1) / BN;
    const uint32_t m_tiles = (M + 32 * MT - 1) / (32 * MT);
    const uint32_t splits_req = layer_forward_q_splits(M, in_features, out_features);
    const uint32_t ksteps = (in_features + BK - 1) / BK;
    const uint32_t rows_per_split = (ksteps + splits_req - 1) / splits_req * BK;
    const uint32_t splits = (in_features + rows_per_split - 1) / rows_per_split;
    const uint32_t jobs = n_tiles * splits * m_tiles;
    const uint32_t padded = (book_bytes + 15) & ~15u;
    if (padded <= kMaxLdsBook) {
        auto kernel = layer_forward_q_kernel<DT, MT, BITS, true>;
        const uint32_t lds = kTileBytes + padded;
        hipError_t e = allow_lds(kernel, lds);
        if (e != hipSuccess) return e;
        const dim3 grid(std::min<uint32_t>(uint32_t(compute_units()), jobs));
        hipLaunchKernelGGL(kernel, grid, dim3(kThreads), lds, s, x, M, qbook, book_bytes, scale, K, g, codes, per_row, in_features,
                           out_features, bias, y, partial, n_tiles, splits, rows_per_split, m_tiles);
    } else {
        const dim3 grid(std::min<uint32_t>(uint32_t(compute_units()) * 4, jobs));
        hipLaunchKernelGGL((layer_forward_q_kernel<DT, MT, BITS, false>), grid, dim3(kThreads), kTileBytes, s, x, M, qbook,
                           book_bytes, scale, K, g, codes, per_row, in_features, out_features, bias, y, partial, n_tiles, splits,
                           rows_per_split, m_tiles);
    }
    if (splits > 1) {
        const uint64_t n = uint64_t(M) * out_features;
        hipLaunchKernelGGL(forward_q_reduce_kernel<DT>, dim3(uint32_t((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, s,
                           partial, n, out_features, splits, scale, bias, y);
    }
    return hipGetLastError();
}

hipError_t launch_layer_forward_q(const void* x, uint32_t M, const void* qbook, int bits, const float* scale, uint32_t K,
                                  uint32_t g, const uint16_t* codes, uint32_t in_features, uint32_t out_features,
                                  const void* bias, void* y, int dtype, float* partial, hipStream_t s)
{
    const uint32_t book_bytes = uint32_t((uint64_t(K) * g * bits + 7) / 8);
    const uint16_t* xs = static_cast<const uint16_t*>(x);
    const uint8_t* qb = static_cast<const uint8_t*>(qbook);
    const uint16_t* bs = static_cast<const uint16_t*>(bias);
    uint16_t* ys = static_cast<uint16_t*>(y);
    if (lds_book_applies(K, g, bits) && M > 16 && M <= 64) {
#define CC_MQ(DT, BITS, G, MT) return forward_q_mfma_t<DT, BITS, G, MT>(xs, M, qb, book_bytes, scale, K, codes, in_features, out_features, bs, ys, partial, s)
#define CC_MQ_MT(DT, BITS, G) do { if (M <= 32) CC_MQ(DT, BITS, G, 1); else CC_MQ(DT, BITS, G, 2); } while (0)
#define CC_MQ_G(DT, BITS) do { if (g == 4) CC_MQ_MT(DT, BITS, 4); else CC_MQ_MT(DT, BITS, 8); } while (0)
        if (dtype == 1 && bits == 4) CC_MQ_G(1, 4);
        if (dtype == 1 && bits == 8) CC_MQ_G(1, 8);
        if (dtype == 2 && bits == 4) CC_MQ_G(2, 4);
        if (dtype == 2 && bits == 8) CC_MQ_G(2, 8);
#undef CC_MQ_G
#undef CC_MQ_MT
#undef CC_MQ
        return hipErrorInvalidValue;
    }
    if (lds_book_applies(K, g, bits) && M <= 16) {
#define CC_GV(DT, BITS, G, MB) return forward_q_gemv_t<DT, BITS, G, MB>(xs, M, qb, book_bytes, scale, K, codes, in_features, out_features, bs, ys, partial, s)
#define CC_GV_MB(DT, BITS, G) do { if (M <= 1) CC_GV(DT, BITS, G, 1); else if (M <= 4) CC_GV(DT, BITS, G, 4); else if (M <= 8) CC_GV(DT, BITS, G, 8); else CC_GV(DT, BITS, G, 16); } while (0)
#define CC_GV_G(DT, BITS) do { if (g == 4) CC_GV_MB(DT, BITS, 4); else CC_GV_MB(DT, BITS, 8); } while (0)
        if (dtype == 1 && bits == 4) CC_GV_G(1, 4);
        if (dtype == 1 && bits == 8) CC_GV_G(1, 8);
        if (dtype == 2 && bits == 4) CC_GV_G(2, 4);
        if (dtype == 2 && bits == 8) CC_GV_G(2, 8);
#undef CC_GV_G
#undef CC_GV_MB
#undef CC_GV
        return hipErrorInvalidValue;
    }
    const int mt = M > 64 ? 4 : (M > 32 ? 2 : 1);
#define CC_FQ(DT, MT, BITS) return forward_q_t<DT, MT, BITS>(xs, M, qb, book_bytes, scale, K, g, codes, in_features, out_features, bs, ys, partial, s)
#define CC_FQ_MT(DT, BITS) do { if (mt == 4) CC_FQ(DT, 4, BITS); else if (mt == 2) CC_FQ(DT, 2, BITS); else CC_FQ(DT, 1, BITS); } while (0)
    if (dtype == 1 && bits == 4) CC_FQ_MT(1, 4);
    if (dtype == 1 && bits == 8) CC_FQ_MT(1, 8);
    if (dtype == 2 && bits == 4) CC_FQ_MT(2, 4);
    if (dtype == 2 && bits == 8) CC_FQ_MT(2, 8);
#undef CC_FQ_MT
#undef CC_FQ
    return hipErrorInvalidValue;
}

}  // namespace cc
