// Forward pass of the compressed linear layer (the paper's layer listing): y = x . W (+ bias), where
// W[in, out] is codebook[codes] with the padding columns cut - but W is never written to memory: each
// workgroup gathers the codebook rows of its tile straight into LDS in matrix-core operand order.
//
// Tiling: a workgroup owns 32*MT rows of x, 64 output columns and a slice of in_features. Per step of 64
// in-features it (1) gathers the 64 x 64 piece of W: one work item = one code column of two neighbouring
// in-features, i.e. two codebook rows, written transposed as 32-bit pairs so that LDS holds Wt[n][k] with
// k contiguous (what the B operand of v_mfma_f32_32x32x16_{bf16,f16} wants: 8 consecutive k per lane);
// (2) each of the 4 waves multiplies its own 16-wide k slice for all of the tile (A operand: 16 bytes of
// an x row per lane, straight from global memory). The four partial tiles are added through LDS at the end.
// The in-feature slices of different workgroups (there to fill the chip when M is small) go to an fp32
// partial buffer and are added in a fixed order by a second kernel: the result does not depend on scheduling.
//
// Bound: one codebook lookup per code per M-tile (L1 tag rate), not HBM: the codes are in*out/g*2 bytes.
#include <algorithm>
#include <type_traits>

#include "common.h"

namespace cc {

namespace {

constexpr int kThreads = 256;
constexpr int BN = 64, BK = 64;
constexpr int S = BK / 2 + 4;  // 32-bit words per Wt row: 16-byte aligned rows, rows 36 words apart

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

template <int DT>
__device__ __forceinline__ float to_f32(uint16_t v)
{
    if constexpr (DT == 1) return float(__builtin_bit_cast(_Float16, v));
    else return __uint_as_float(uint32_t(v) << 16);
}

template <int DT>
__device__ __forceinline__ uint16_t from_f32(float v)
{
    if constexpr (DT == 1) {
        return __builtin_bit_cast(uint16_t, _Float16(v));  // round to nearest even
    } else {
        const uint32_t b = __float_as_uint(v);
        if ((b & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;
        return uint16_t((b + 0x7fffu + ((b >> 16) & 1u)) >> 16);
    }
}

// Row `k` of a codebook of 16-bit elements as 32-bit words (element j in word j/2, half j%2).
__device__ __forceinline__ void load_row_words(const uint16_t* __restrict__ codebook, uint32_t k, uint32_t g, uint32_t (&w)[8])
{
    const uint16_t* row = codebook + size_t(k) * g;
    if (g == 4) {
        const uint2 t = *reinterpret_cast<const uint2*>(row);
        w[0] = t.x; w[1] = t.y;
    } else if (g == 8) {
        const uint4 t = *reinterpret_cast<const uint4*>(row);
        w[0] = t.x; w[1] = t.y; w[2] = t.z; w[3] = t.w;
    } else if (g == 16) {
        const uint4 t = reinterpret_cast<const uint4*>(row)[0], u = reinterpret_cast<const uint4*>(row)[1];
        w[0] = t.x; w[1] = t.y; w[2] = t.z; w[3] = t.w; w[4] = u.x; w[5] = u.y; w[6] = u.z; w[7] = u.w;
    } else if ((g & 1) == 0) {
#pragma unroll
        for (uint32_t q = 0; q < 8; ++q)
            if (2 * q < g) w[q] = reinterpret_cast<const uint32_t*>(row)[q];
    } else {
#pragma unroll
        for (uint32_t q = 0; q < 8; ++q) {
            if (2 * q >= g) break;
            const uint32_t lo = row[2 * q];
            const uint32_t hi = 2 * q + 1 < g ? row[2 * q + 1] : 0u;
            w[q] = lo | (hi << 16);
        }
    }
}

// grid.x = n_tiles * splits (remapped so that one XCD works on neighbouring column tiles, which share the
// cache lines of the codes), grid.y = M tiles.
template <int DT, int MT>
__global__ __launch_bounds__(kThreads) void layer_forward_kernel(
    const uint16_t* __restrict__ x, uint32_t M, const uint16_t* __restrict__ codebook, uint32_t K, uint32_t g,
    const uint16_t* __restrict__ codes, uint32_t per_row, uint32_t in_features, uint32_t out_features,
    const uint16_t* __restrict__ bias, uint16_t* __restrict__ y, float* __restrict__ partial, uint32_t n_tiles,
    uint32_t splits, uint32_t rows_per_split)
{
    __shared__ __attribute__((aligned(16))) uint32_t Wt[BN * S];
    __shared__ float red[4][16][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, h = lane >> 5;

    // column tile and in-feature slice of this workgroup: consecutive workgroup ids go to different XCDs,
    // so give XCD q the q-th contiguous share of the column tiles
    const uint32_t total = n_tiles * splits;
    uint32_t job = blockIdx.x;
    if (total % 8 == 0) job = (blockIdx.x % 8) * (total / 8) + blockIdx.x / 8;
    const uint32_t nt = job / splits, split = job % splits;
    const uint32_t n_lo = nt * BN;
    const uint32_t m0 = blockIdx.y * (32 * MT);
    const uint32_t k_begin = split * rows_per_split, k_end = min(k_begin + rows_per_split, in_features);

    const uint32_t cn_lo = n_lo / g;
    const uint32_t cn_hi = min((n_lo + BN - 1) / g, per_row - 1);
    const uint32_t cpr = cn_hi - cn_lo + 1;   // code columns that touch this tile
    const uint32_t items = (BK / 2) * cpr;    // (pair of in-features, code column)

    f32x16 acc[MT][2];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][nb][r] = 0.0f;

    for (uint32_t k0 = k_begin; k0 < k_end; k0 += BK) {
        // ---- gather the W piece: Wt[n - n_lo][k - k0], two k per 32-bit word
        for (uint32_t it = threadIdx.x; it < items; it += kThreads) {
            const uint32_t rp = it / cpr, c = it % cpr;
            const uint32_t r0 = k0 + 2 * rp, r1 = r0 + 1;
            const uint32_t code0 = r0 < k_end ? min(uint32_t(codes[size_t(r0) * per_row + cn_lo + c]), K - 1) : 0u;
            const uint32_t code1 = r1 < k_end ? min(uint32_t(codes[size_t(r1) * per_row + cn_lo + c]), K - 1) : 0u;
            // the two codebook rows, fetched with the widest loads their alignment allows (one L1 lookup per
            // load instruction and lane is what bounds this kernel)
            uint32_t w0[8], w1[8];  // up to 16 elements each, two per word
            load_row_words(codebook, code0, g, w0);
            load_row_words(codebook, code1, g, w1);
            const bool live0 = r0 < k_end, live1 = r1 < k_end;
            const int nbase = int((cn_lo + c) * g) - int(n_lo);
#pragma unroll
            for (uint32_t j = 0; j < 16; ++j) {
                if (j >= g) break;
                const int n = nbase + int(j);
                if (n < 0 || n >= BN) continue;
                const uint32_t e0 = live0 ? (w0[j >> 1] >> (16 * (j & 1))) & 0xffffu : 0u;
                const uint32_t e1 = live1 ? (w1[j >> 1] >> (16 * (j & 1))) & 0xffffu : 0u;
                Wt[n * S + rp] = e0 | (e1 << 16);
            }
        }
        __syncthreads();
        // ---- this wave's 16-wide k slice of the step
        const uint32_t kk = k0 + 16 * wave + 8 * h;  // first of this lane's 8 in-features
        u32x4 b[2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
            b[nb] = *reinterpret_cast<const u32x4*>(&Wt[(32 * nb + (lane & 31)) * S + 8 * wave + 4 * h]);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const uint32_t m = m0 + 32 * mt + (lane & 31);
            u32x4 a = {0u, 0u, 0u, 0u};
            if (m < M && kk < k_end) a = *reinterpret_cast<const u32x4*>(x + size_t(m) * in_features + kk);
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) acc[mt][nb] = mma<DT>(a, b[nb], acc[mt][nb]);
        }
        __syncthreads();
    }

    // ---- add the four k slices of the workgroup, then store
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) red[wave][r][lane] = acc[mt][nb][r];
            __syncthreads();
            // wave v finishes accumulator registers 4v .. 4v+3 of all 64 lanes
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int r = 4 * wave + q;
                const float v = ((red[0][r][lane] + red[1][r][lane]) + red[2][r][lane]) + red[3][r][lane];
                const uint32_t m = m0 + 32 * mt + (r & 3) + 8 * (r >> 2) + 4 * h;
                const uint32_t n = n_lo + 32 * nb + (lane & 31);
                if (m < M && n < out_features) {
                    if (splits == 1) {
                        y[size_t(m) * out_features + n] = from_f32<DT>(bias ? v + to_f32<DT>(bias[n]) : v);
                    } else {
                        partial[(size_t(split) * M + m) * out_features + n] = v;
                    }
                }
            }
            __syncthreads();
        }
    }
}

template <int DT>
__global__ __launch_bounds__(kThreads) void layer_forward_reduce_kernel(const float* __restrict__ partial, uint64_t n,
                                                                        uint32_t out_features, uint32_t splits,
                                                                        const uint16_t* __restrict__ bias,
                                                                        uint16_t* __restrict__ y)
{
    const uint64_t t = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
    if (t >= n) return;
    float v = partial[t];
    for (uint32_t s = 1; s < splits; ++s) v += partial[uint64_t(s) * n + t];  // fixed order
    if (bias) v += to_f32<DT>(bias[t % out_features]);
    y[t] = from_f32<DT>(v);
}

// ---- few rows of x (decode-time M <= 4), g = 4 ------------------------------------------------------------------
// No matrix cores and no transposed tile: with one row of x a 32-row matrix instruction is 97 % idle, and what bounds
// the pass is the one codebook lookup per code. A lane owns one code column (g outputs) and walks down the
// in-features of its slice: per pair of in-features it reads the two codes (the 64 lanes of a wave read 128
// contiguous bytes per row), looks both codebook rows up (one 8- or 16-byte load each, L2-resident), converts them
// and does MB * g * 2 fused multiply-adds against x values that are uniform over the wave (scalar loads). The 8
// waves of a workgroup share 64 code columns and take every 8th pair; their partial sums meet in LDS in a fixed
// order, the slices of in_features in a second kernel in a fixed order: same inputs, same bits.
// Measured at 4096 x 11008, K = 65536: 58 us for M = 1..4 against 65 us for the tile kernel above (4096 x 4096: 27-29
// against 30 us); the lookups (L1 misses served by L2, about 1.5 clocks each per compute unit) bound both. With 8
// rows of x per lane the two are level (61 / 64 us and 31 / 30 us), with 16 the registers halve the occupancy (74 us),
// and at g = 8 there is no gain at any M: those stay with the tile kernel.
constexpr int kFewThreads = 512, kFewWaves = 8, kFewCols = 64;
constexpr uint32_t kFewMaxSplits = 64;

template <int DT, int G, int MB>
__global__ __launch_bounds__(kFewThreads) void layer_forward_few_kernel(
    const uint16_t* __restrict__ x, uint32_t M, const uint16_t* __restrict__ codebook, uint32_t K,
    const uint16_t* __restrict__ codes, uint32_t per_row, uint32_t in_features, uint32_t out_features,
    const uint16_t* __restrict__ bias, uint16_t* __restrict__ y, float* __restrict__ partial, uint32_t col_blocks,
    uint32_t splits, uint32_t rows_per_split)
{
    constexpr int MC = G == 4 ? 2 : 1;                      // rows of x per reduction round (16 KB of LDS)
    __shared__ float red[kFewWaves * MC * kFewCols * G];    // [wave][mc][column * G + j]
    const int lane = threadIdx.x & 63;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t cb = blockIdx.x % col_blocks, split = blockIdx.x / col_blocks;
    const uint32_t cn = cb * kFewCols + lane;
    const bool live = cn < per_row;
    const uint32_t k_begin = split * rows_per_split, k_end = min(k_begin + rows_per_split, in_features);
    typedef typename std::conditional<G == 4, uint2, uint4>::type Row;
    const Row* rows = reinterpret_cast<const Row*>(codebook);

    float acc[MB][G];
#pragma unroll
    for (int m = 0; m < MB; ++m)
#pragma unroll
        for (int j = 0; j < G; ++j) acc[m][j] = 0.0f;

    // pairs of in-features (rows 2p, 2p + 1): this wave takes p = k_begin / 2 + wave, + 8, ...; the codes of U pairs
    // are requested, then their 2 U codebook rows, before any is used; in_features is even, so is every k_begin
    constexpr int U = 8;
    for (uint32_t p0 = k_begin / 2 + wave; 2 * p0 < k_end; p0 += kFewWaves * U) {
        uint32_t c0[U], c1[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t p = p0 + u * kFewWaves;
            const bool on = live && 2 * p < k_end;
            c0[u] = on ? uint32_t(codes[size_t(2 * p) * per_row + cn]) : 0u;
            c1[u] = on ? uint32_t(codes[size_t(2 * p + 1) * per_row + cn]) : 0u;
        }
        Row r0[U], r1[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            r0[u] = rows[min(c0[u], K - 1)];
            r1[u] = rows[min(c1[u], K - 1)];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t p = p0 + u * kFewWaves;
            if (2 * p >= k_end) break;  // wave-uniform
            uint32_t w0[G / 2], w1[G / 2];
            if constexpr (G == 4) {
                w0[0] = r0[u].x; w0[1] = r0[u].y; w1[0] = r1[u].x; w1[1] = r1[u].y;
            } else {
                w0[0] = r0[u].x; w0[1] = r0[u].y; w0[2] = r0[u].z; w0[3] = r0[u].w;
                w1[0] = r1[u].x; w1[1] = r1[u].y; w1[2] = r1[u].z; w1[3] = r1[u].w;
            }
            float f0[G], f1[G];
#pragma unroll
            for (int q = 0; q < G / 2; ++q) {
                f0[2 * q] = to_f32<DT>(uint16_t(w0[q] & 0xffffu));
                f0[2 * q + 1] = to_f32<DT>(uint16_t(w0[q] >> 16));
                f1[2 * q] = to_f32<DT>(uint16_t(w1[q] & 0xffffu));
                f1[2 * q + 1] = to_f32<DT>(uint16_t(w1[q] >> 16));
            }
#pragma unroll
            for (int m = 0; m < MB; ++m) {
                // both x values of the pair in one (wave-uniform) 32-bit load
                const uint32_t xw = m < int(M) ? reinterpret_cast<const uint32_t*>(x + size_t(m) * in_features)[p] : 0u;
                const float x0 = to_f32<DT>(uint16_t(xw & 0xffffu)), x1 = to_f32<DT>(uint16_t(xw >> 16));
#pragma unroll
                for (int j = 0; j < G; ++j) {
                    acc[m][j] = __builtin_fmaf(x0, f0[j], acc[m][j]);
                    acc[m][j] = __builtin_fmaf(x1, f1[j], acc[m][j]);
                }
            }
        }
    }

    // sum over the 8 waves, MC rows of x per round: thread t finishes element t of the round
#pragma unroll
    for (int m0 = 0; m0 < MB; m0 += MC) {
        __syncthreads();
#pragma unroll
        for (int mc = 0; mc < MC; ++mc)
#pragma unroll
            for (int j = 0; j < G; ++j)
                if (m0 + mc < MB) red[((wave * MC + mc) * kFewCols + lane) * G + j] = acc[(m0 + mc) % MB][j];
        __syncthreads();
        constexpr int kRound = MC * kFewCols * G;  // elements per round
        for (int t = threadIdx.x; t < kRound; t += kFewThreads) {
            const int mc = t / (kFewCols * G), rest = t % (kFewCols * G);
            float v = 0.0f;
#pragma unroll
            for (int w = 0; w < kFewWaves; ++w) v += red[(w * MC + mc) * kFewCols * G + rest];
            const uint32_t m = m0 + mc;
            const uint32_t n = cb * kFewCols * G + rest;
            if (m < M && m < MB && n < out_features) {
                if (splits == 1) {
                    y[size_t(m) * out_features + n] = from_f32<DT>(bias ? v + to_f32<DT>(bias[n]) : v);
                } else {
                    partial[(size_t(split) * M + m) * out_features + n] = v;
                }
            }
        }
    }
}

// Slices of in_features for the few-rows kernel: about four workgroups per compute unit, at least four pairs of
// in-features per wave.
uint32_t few_rows_splits(uint32_t in_features, uint32_t per_row)
{
    const uint32_t col_blocks = (per_row + kFewCols - 1) / kFewCols;
    uint32_t splits = (4 * 256 + col_blocks - 1) / col_blocks;
    splits = std::min<uint32_t>(splits, std::max<uint32_t>(1, in_features / (2 * kFewWaves * 4)));
    return std::max<uint32_t>(1, std::min<uint32_t>(splits, kFewMaxSplits));
}

template <int DT, int G, int MB>
void forward_few_t(const uint16_t* x, uint32_t M, const uint16_t* codebook, uint32_t K, const uint16_t* codes,
                   uint32_t in_features, uint32_t out_features, const uint16_t* bias, uint16_t* y, float* partial,
                   hipStream_t s)
{
    const uint32_t per_row = (out_features + G - 1) / G;
    const uint32_t col_blocks = (per_row + kFewCols - 1) / kFewCols;
    const uint32_t req = few_rows_splits(in_features, per_row);
    // slices hold whole groups of 16 in-features (one pair per wave), so that every slice starts at wave 0's pair
    const uint32_t groups = (in_features + 2 * kFewWaves - 1) / (2 * kFewWaves);
    const uint32_t rows_per_split = (groups + req - 1) / req * (2 * kFewWaves);
    const uint32_t splits = (in_features + rows_per_split - 1) / rows_per_split;
    hipLaunchKernelGGL((layer_forward_few_kernel<DT, G, MB>), dim3(col_blocks * splits), dim3(kFewThreads), 0, s, x, M, codebook, K,
                       codes, per_row, in_features, out_features, bias, y, partial, col_blocks, splits, rows_per_split);
    if (splits > 1) {
        const uint64_t n = uint64_t(M) * out_features;
        hipLaunchKernelGGL(layer_forward_reduce_kernel<DT>, dim3(uint32_t((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, s,
                           partial, n, out_features, splits, bias, y);
    }
}

template <int DT, int G>
void forward_few_rows(const uint16_t* x, uint32_t M, const uint16_t* codebook, uint32_t K, const uint16_t* codes,
                      uint32_t in_features, uint32_t out_features, const uint16_t* bias, uint16_t* y, float* partial,
                      hipStream_t s)
{
#define CC_FEW(MB) forward_few_t<DT, G, MB>(x, M, codebook, K, codes, in_features, out_features, bias, y, partial, s)
    if (M == 1) CC_FEW(1); else if (M == 2) CC_FEW(2); else CC_FEW(4);
#undef CC_FEW
}

template <int DT, int MT>
void forward_t(const uint16_t* x, uint32_t M, const uint16_t* codebook, uint32_t K, uint32_t g, const uint16_t* codes,
               uint32_t in_features, uint32_t out_features, const uint16_t* bias, uint16_t* y, float* partial,
               uint32_t splits, uint32_t rows_per_split, hipStream_t s)
{
    const uint32_t per_row = (out_features + g - 1) / g;
    const uint32_t n_tiles = (out_features + BN - 1) / BN;
    const dim3 grid(n_tiles * splits, (M + 32 * MT - 1) / (32 * MT));
    hipLaunchKernelGGL((layer_forward_kernel<DT, MT>), grid, dim3(kThreads), 0, s, x, M, codebook, K, g, codes, per_row,
                       in_features, out_features, bias, y, partial, n_tiles, splits, rows_per_split);
    if (splits > 1) {
        const uint64_t n = uint64_t(M) * out_features;
        hipLaunchKernelGGL(layer_forward_reduce_kernel<DT>, dim3(uint32_t((n + kThreads - 1) / kThreads)), dim3(kThreads), 0, s,
                           partial, n, out_features, splits, bias, y);
    }
}

}  // namespace

// Whether a call takes the few-rows kernel, and the most in-feature slices that kernel uses (sizes the partial buffer
// when the sub-vector length is not known).
bool layer_forward_few_rows(uint64_t M, uint32_t g) { return M <= 4 && g == 4; }
uint32_t layer_forward_few_rows_max_splits() { return kFewMaxSplits; }

// How many in-feature slices a call uses (also sizes the partial buffer): enough workgroups to fill the chip.
uint32_t layer_forward_splits(uint64_t M, uint32_t in_features, uint32_t out_features)
{
    const uint64_t n_tiles = (out_features + BN - 1) / BN;
    const int mt = M > 64 ? 4 : (M > 32 ? 2 : 1);
    const uint64_t m_tiles = (M + 32 * mt - 1) / (32 * mt);
    const uint64_t ksteps = (in_features + BK - 1) / BK;
    uint64_t splits = (1024 + n_tiles * m_tiles - 1) / (n_tiles * m_tiles);
    splits = std::min<uint64_t>(splits, std::max<uint64_t>(1, ksteps / 2));  // at least two steps per slice
    return uint32_t(std::max<uint64_t>(1, std::min<uint64_t>(splits, 64)));
}

hipError_t launch_layer_forward(const void* x, uint32_t M, const void* codebook, int dtype, uint32_t K, uint32_t g,
                                const uint16_t* codes, uint32_t in_features, uint32_t out_features, const void* bias,
                                void* y, float* partial, hipStream_t s)
{
    const uint16_t* xs = static_cast<const uint16_t*>(x);
    const uint16_t* cb = static_cast<const uint16_t*>(codebook);
    const uint16_t* bs = static_cast<const uint16_t*>(bias);
    uint16_t* ys = static_cast<uint16_t*>(y);
    if (layer_forward_few_rows(M, g)) {
        if (dtype != 1 && dtype != 2) return hipErrorInvalidValue;
        if (dtype == 1) forward_few_rows<1, 4>(xs, M, cb, K, codes, in_features, out_features, bs, ys, partial, s);
        else forward_few_rows<2, 4>(xs, M, cb, K, codes, in_features, out_features, bs, ys, partial, s);
        return hipGetLastError();
    }
    const uint32_t splits = layer_forward_splits(M, in_features, out_features);
    const uint32_t ksteps = (in_features + BK - 1) / BK;
    const uint32_t rows_per_split = (ksteps + splits - 1) / splits * BK;
    const uint32_t used = (in_features + rows_per_split - 1) / rows_per_split;  // slices that are not empty
    const int mt = M > 64 ? 4 : (M > 32 ? 2 : 1);
#define CC_FWD(DT, MT) forward_t<DT, MT>(xs, M, cb, K, g, codes, in_features, out_features, bs, ys, partial, used, rows_per_split, s)
    if (dtype == 1) {
        if (mt == 4) CC_FWD(1, 4); else if (mt == 2) CC_FWD(1, 2); else CC_FWD(1, 1);
    } else if (dtype == 2) {
        if (mt == 4) CC_FWD(2, 4); else if (mt == 2) CC_FWD(2, 2); else CC_FWD(2, 1);
    } else {
        return hipErrorInvalidValue;
    }
#undef CC_FWD
    return hipGetLastError();
}

}  // namespace cc
