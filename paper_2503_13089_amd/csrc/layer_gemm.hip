// Forward pass of the compressed linear layer at prefill-sized batches (the paper's layer listing: rebuild the
// weight from (codebook, codes), then y = x . W + bias), as two hand-written kernels:
//
//   1. layer_weight_t_kernel: the listing's gather, written TRANSPOSED: Wt[n][k] = codebook[code(k, n)][n % g], so
//      that both operands of the product are contiguous along the contraction index, which is what the matrix
//      cores' operand registers want (8 consecutive k per lane). 64 x 64 tiles through LDS: codes are read along a
//      row of W, Wt is written along its own rows, both in full cache lines.
//   2. gemm_tn_kernel: y[M][N] = x[M][K] . Wt[N][K]^T on v_mfma_f32_32x32x16_{bf16,f16}. A workgroup of 4 waves owns
//      a 256 x 128 tile of y (each wave 128 x 64 = 4 x 2 accumulator tiles of 32 x 32, held in registers for the
//      whole contraction), steps through K in slices of 64, and stages both operand slices in LDS, double-buffered:
//      the next slice travels global -> registers while the current one is multiplied, then registers -> LDS, one
//      barrier per slice. LDS rows are padded to 72 halves (36 words) so that the 16-byte fragment reads of a
//      half-wave fall on 16 different bank quads. Products of two 16-bit values are exact in fp32; the sum is fp32
//      in a fixed order; bias (and, for the quantised codebook, the scale) are applied to the finished sum and y is
//      rounded once.
//      Workgroups are numbered so that one XCD (they are dealt to the 8 XCDs in turn) works on neighbouring column
//      panels with all row panels of x: its L2 then holds the Wt panels it is using, and x comes once per XCD.
//      Few tiles (M of a few hundred): the contraction is also split over workgroups, fp32 partial tiles go to the
//      workspace and a second kernel adds them in a fixed order - the result never depends on scheduling.
//
// Bound: the bf16 / fp16 matrix cores (2 M N K flop against 2.5 PFLOP/s); the rebuild is HBM-bound (2 bytes written
// per weight).
#include <algorithm>

#include "common.h"

namespace cc {

namespace {

constexpr int kThreads = 256;
constexpr int BM = 256, BN = 128, BK = 32;
constexpr int LDT = BK + 8;                 // halves per LDS row (20 words: the 16-byte reads of 16 lanes hit 16 bank quads)
constexpr int kStageHalves = (BM + BN) * LDT;
constexpr uint32_t kGemmLdsBytes = 2 * kStageHalves * 2;   // 61,440 bytes: two workgroups per CU

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

// ---- 1. transposed rebuild: Wt[n][k], n < out_features, k < in_features, row length ldk = in_features
// Three steps per 64 x 64 tile: the tile's codes (64 rows of W, the code columns that touch the tile) go to LDS with
// reads along the rows of the code matrix; then a wave takes one code column and its 64 lanes the 64 rows, so that
// the elements they write into the transposed tile are neighbours in LDS (lanes along n would hit the same banks);
// then the tile leaves in 16-byte pieces along k.
constexpr int kWtTile = 64;
constexpr int kWtMaxCols = kWtTile + 2;  // code columns touching a tile: at most 64 / g + 2 <= 66 for g >= 1
__global__ __launch_bounds__(kThreads) void layer_weight_t_kernel(const uint16_t* __restrict__ codebook, uint32_t K, uint32_t g,
                                                                  const uint16_t* __restrict__ codes, uint32_t per_row,
                                                                  uint32_t in_features, uint32_t out_features,
                                                                  uint16_t* __restrict__ wt)
{
    constexpr int T = kWtTile, LT = T + 8;
    __shared__ __attribute__((aligned(16))) uint16_t tile[T * LT];  // [n][k]
    __shared__ uint16_t ctile[T * kWtMaxCols];                      // [k][code column]
    const uint32_t n_lo = blockIdx.x * T, k0 = blockIdx.y * T;
    const uint32_t cn_lo = n_lo / g;
    const uint32_t cn_hi = min((n_lo + T - 1) / g, per_row - 1);
    const uint32_t cpr = cn_hi - cn_lo + 1;  // code columns that touch this tile
    const uint32_t items = T * cpr;
    for (uint32_t it = threadIdx.x; it < items; it += kThreads) {
        const uint32_t kr = it / cpr, c = it % cpr;
        const uint32_t k = min(k0 + kr, in_features - 1);  // rows past the edge are never stored
        ctile[kr * cpr + c] = codes[size_t(k) * per_row + cn_lo + c];
    }
    __syncthreads();
    for (uint32_t it = threadIdx.x; it < items; it += kThreads) {
        const uint32_t c = it / T, kr = it % T;
        const uint32_t code = min(uint32_t(ctile[kr * cpr + c]), K - 1);
        const uint16_t* row = codebook + size_t(code) * g;
        const int nbase = int((cn_lo + c) * g) - int(n_lo);
        if (g == 4) {
            const uint2 r = *reinterpret_cast<const uint2*>(row);
            const uint16_t e[4] = {uint16_t(r.x), uint16_t(r.x >> 16), uint16_t(r.y), uint16_t(r.y >> 16)};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n = nbase + j;
                if (n >= 0 && n < T) tile[n * LT + kr] = e[j];
            }
        } else if (g == 8) {
            const uint4 r = *reinterpret_cast<const uint4*>(row);
            const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int n = nbase + j;
                if (n >= 0 && n < T) tile[n * LT + kr] = uint16_t(w[j >> 1] >> (16 * (j & 1)));
            }
        } else {
            for (uint32_t j = 0; j < g; ++j) {
                const int n = nbase + int(j);
                if (n >= 0 && n < T) tile[n * LT + kr] = row[j];
            }
        }
    }
    __syncthreads();
    // 16-byte pieces along k: 8 threads write the 128 bytes of one row of the tile
#pragma unroll
    for (int pass = 0; pass < T * 8 / kThreads; ++pass) {
        const uint32_t n = pass * (kThreads / 8) + threadIdx.x / 8, kc = (threadIdx.x % 8) * 8;
        if (n_lo + n < out_features && k0 + kc < in_features)  // in_features is a multiple of 8: whole pieces
            *reinterpret_cast<uint4*>(wt + size_t(n_lo + n) * in_features + k0 + kc) =
                *reinterpret_cast<const uint4*>(&tile[n * LT + kc]);
    }
}

// Plain transpose of a 16-bit matrix, W[rows][cols] -> Wt[cols][rows] (rows a multiple of 8), 64 x 64 tiles.
__global__ __launch_bounds__(kThreads) void transpose16_kernel(const uint16_t* __restrict__ w, uint32_t rows, uint32_t cols,
                                                               uint16_t* __restrict__ wt)
{
    constexpr int T = 64, LT = T + 8;
    __shared__ __attribute__((aligned(16))) uint16_t tile[T * LT];  // [col][row]
    const uint32_t c0 = blockIdx.x * T, r0 = blockIdx.y * T;
    for (uint32_t e = threadIdx.x; e < T * T; e += kThreads) {
        const uint32_t r = e / T, c = e % T;
        if (r0 + r < rows && c0 + c < cols) tile[c * LT + r] = w[size_t(r0 + r) * cols + c0 + c];
    }
    __syncthreads();
#pragma unroll
    for (int pass = 0; pass < T * 8 / kThreads; ++pass) {
        const uint32_t c = pass * (kThreads / 8) + threadIdx.x / 8, rc = (threadIdx.x % 8) * 8;
        if (c0 + c < cols && r0 + rc < rows)
            *reinterpret_cast<uint4*>(wt + size_t(c0 + c) * rows + r0 + rc) = *reinterpret_cast<const uint4*>(&tile[c * LT + rc]);
    }
}

// ---- 2. the product
// Jobs: the tiles of y in whole rounds of the chip's workgroup slots take the full contraction and write y themselves
// (`whole` of them); the tiles of the last, partial round are each cut into f in-feature slices, so that the round
// is short and full instead of long and half empty, and leave fp32 partial tiles for gemm_finish_kernel. The cut
// depends on the shape alone.
template <int DT>
__global__ __launch_bounds__(kThreads, 2) void gemm_tn_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ wt,
                                                              uint32_t M, uint32_t N, uint32_t K,
                                                              const float* __restrict__ scale,
                                                              const uint16_t* __restrict__ bias, uint16_t* __restrict__ y,
                                                              float* __restrict__ partial, uint32_t m_tiles, uint32_t whole,
                                                              uint32_t f, uint32_t k_per_split, uint32_t jobs)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, h = lane >> 5, l32 = lane & 31;
    const int wm = wave & 1, wn = wave >> 1;

    // job of this workgroup: XCD q (= blockIdx % 8) takes the q-th contiguous share of the whole tiles and then the q-th share of the slices of the cut tiles; within a share the row panels of x vary fastest, so
    // neighbours share a panel of Wt
    const uint32_t xcd = blockIdx.x % 8, local = blockIdx.x / 8;
    const uint32_t whole_per = (whole + 7) / 8, cut_per = (jobs - whole + 7) / 8;
    uint32_t job;
    if (local < whole_per) {
        job = xcd * whole_per + local;
        if (job >= whole) return;
    } else {
        job = whole + xcd * cut_per + (local - whole_per);
        if (local - whole_per >= cut_per || job >= jobs) return;
    }
    const bool direct = job < whole;
    const uint32_t cut = direct ? 0u : (job - whole) / f;   // which tile of the partial round
    const uint32_t split = direct ? 0u : (job - whole) % f;
    const uint32_t tile = direct ? job : whole + cut;
    const uint32_t mt = tile % m_tiles, nt = tile / m_tiles;
    const uint32_t m0 = mt * BM, n0 = nt * BN;
    const uint32_t k_begin = direct ? 0u : split * k_per_split;
    const uint32_t k_end = direct ? K : min(k_begin + k_per_split, K);

    // global -> register staging: 16-byte pieces, BK / 8 per operand row and slice; thread t takes piece t % PR of
    // rows t / PR + RP i. Rows past the edge are clamped (their results are never stored); a piece past k_end is
    // read from the last valid piece of its row instead and replaced by zeros (K and k_per_split are multiples of 8).
    constexpr int PR = BK / 8, RP = kThreads / PR, NA = BM / RP, NB = BN / RP;
    const uint32_t prow = threadIdx.x / PR, pk = (threadIdx.x % PR) * 8;
    const uint16_t* a_src[NA];
    const uint16_t* b_src[NB];
#pragma unroll
    for (int i = 0; i < NA; ++i) a_src[i] = x + size_t(min(m0 + prow + RP * i, M - 1)) * K;
#pragma unroll
    for (int i = 0; i < NB; ++i) b_src[i] = wt + size_t(min(n0 + prow + RP * i, N - 1)) * K;
    uint4 a_reg[NA], b_reg[NB];
    auto fetch = [&](uint32_t k0) {
        const bool live = k0 + pk < k_end;
        const uint32_t k = live ? k0 + pk : K - 8;
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const uint4 v = *reinterpret_cast<const uint4*>(a_src[i] + k);
            a_reg[i] = live ? v : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const uint4 v = *reinterpret_cast<const uint4*>(b_src[i] + k);
            b_reg[i] = live ? v : make_uint4(0, 0, 0, 0);
        }
    };
    auto stash = [&](int buf) {
        uint16_t* As = lds + buf * kStageHalves;
        uint16_t* Bs = As + BM * LDT;
#pragma unroll
        for (int i = 0; i < NA; ++i) *reinterpret_cast<uint4*>(&As[(prow + RP * i) * LDT + pk]) = a_reg[i];
#pragma unroll
        for (int i = 0; i < NB; ++i) *reinterpret_cast<uint4*>(&Bs[(prow + RP * i) * LDT + pk]) = b_reg[i];
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    fetch(k_begin);
    stash(0);
    __syncthreads();
    int cur = 0;
    for (uint32_t k0 = k_begin; k0 < k_end; k0 += BK) {
        const bool more = k0 + BK < k_end;
        if (more) fetch(k0 + BK);
        const uint16_t* As = lds + cur * kStageHalves + (wm * 128 + l32) * LDT + 8 * h;
        const uint16_t* Bs = lds + cur * kStageHalves + BM * LDT + (wn * 64 + l32) * LDT + 8 * h;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            u32x4 a[4], b[2];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = *reinterpret_cast<const u32x4*>(As + 32 * i * LDT + 16 * kk);
#pragma unroll
            for (int j = 0; j < 2; ++j) b[j] = *reinterpret_cast<const u32x4*>(Bs + 32 * j * LDT + 16 * kk);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = mma<DT>(a[i], b[j], acc[i][j]);
        }
        if (more) stash(cur ^ 1);
        __syncthreads();
        cur ^= 1;
    }

    // ---- epilogue: accumulator register r of lane (l32, h) is row r % 4 + 8 (r / 4) + 4 h, column l32 of its tile
    const float sc = (direct && scale != nullptr) ? *scale : 1.0f;
    float* ptile = partial + (size_t(cut) * f + split) * (BM * BN);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint32_t nl = wn * 64 + 32 * j + l32, n = n0 + nl;
            if (n >= N) continue;
            const float bv = (direct && bias != nullptr) ? to_f32<DT>(bias[n]) : 0.0f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const uint32_t ml = wm * 128 + 32 * i + (r & 3) + 8 * (r >> 2) + 4 * h, m = m0 + ml;
                if (m >= M) continue;
                if (direct) {
                    float v = acc[i][j][r];
                    if (scale != nullptr) v *= sc;
                    if (bias != nullptr) v += bv;
                    y[size_t(m) * N + n] = from_f32<DT>(v);
                } else {
                    ptile[ml * BN + nl] = acc[i][j][r];
                }
            }
        }
}

// The tiles of the partial round: y = round(scale * (sum of the f slices, in order) + bias); scale may be NULL (= 1)
template <int DT>
__global__ __launch_bounds__(kThreads) void gemm_finish_kernel(const float* __restrict__ partial, uint32_t M, uint32_t N,
                                                               uint32_t m_tiles, uint32_t whole, uint32_t f,
                                                               const float* __restrict__ scale,
                                                               const uint16_t* __restrict__ bias, uint16_t* __restrict__ y)
{
    const uint32_t cut = blockIdx.y, tile = whole + cut;
    const uint32_t m0 = (tile % m_tiles) * BM, n0 = (tile / m_tiles) * BN;
    const uint32_t e = blockIdx.x * kThreads + threadIdx.x;  // element of the tile
    const uint32_t ml = e / BN, nl = e % BN, m = m0 + ml, n = n0 + nl;
    if (m >= M || n >= N) return;
    const float* p = partial + size_t(cut) * f * (BM * BN) + e;
    float v = p[0];
    for (uint32_t s = 1; s < f; ++s) v += p[size_t(s) * (BM * BN)];
    if (scale != nullptr) v *= *scale;
    if (bias != nullptr) v += to_f32<DT>(bias[n]);
    y[size_t(m) * N + n] = from_f32<DT>(v);
}

// Workgroups the chip holds at once: 256 compute units, two workgroups each (their LDS and registers allow two).
constexpr uint32_t kGemmSlots = 512;

struct GemmShape {
    uint32_t m_tiles, n_tiles, whole, cut_tiles, f, k_per_split, jobs;
};

GemmShape gemm_shape(uint64_t M, uint32_t K, uint32_t N)
{
    GemmShape s;
    s.m_tiles = uint32_t((M + BM - 1) / BM);
    s.n_tiles = (N + BN - 1) / BN;
    const uint32_t tiles = s.m_tiles * s.n_tiles;
    const uint32_t ksteps = (K + BK - 1) / BK;
    s.cut_tiles = tiles % kGemmSlots;
    s.whole = tiles - s.cut_tiles;
    uint32_t f = 1;
    if (s.cut_tiles > 0) f = std::max(1u, std::min({kGemmSlots / s.cut_tiles, std::max(1u, ksteps / 8), 16u}));
    s.k_per_split = (ksteps + f - 1) / f * BK;
    s.f = (K + s.k_per_split - 1) / s.k_per_split;  // slices that are not empty
    if (s.f == 1) {  // nothing to gain from a cut: every tile takes the whole contraction
        s.whole = tiles;
        s.cut_tiles = 0;
    }
    s.jobs = s.whole + s.cut_tiles * s.f;
    return s;
}

}  // namespace

// fp32 partial tiles the product needs in the workspace (0 if every tile writes y directly)
size_t layer_gemm_partial_bytes(uint64_t M, uint32_t in_features, uint32_t out_features)
{
    const GemmShape s = gemm_shape(M, in_features, out_features);
    return align256(size_t(s.cut_tiles) * s.f * BM * BN * 4);
}

hipError_t launch_layer_weight_t(const void* codebook, uint32_t K, uint32_t g, const uint16_t* codes, uint32_t in_features,
                                 uint32_t out_features, void* wt, hipStream_t s)
{
    const uint32_t per_row = (out_features + g - 1) / g;
    const dim3 grid((out_features + 63) / 64, (in_features + 63) / 64);
    if (grid.y > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(layer_weight_t_kernel, grid, dim3(kThreads), 0, s, static_cast<const uint16_t*>(codebook), K, g, codes,
                       per_row, in_features, out_features, static_cast<uint16_t*>(wt));
    return hipGetLastError();
}

hipError_t launch_transpose16(const void* w, uint32_t rows, uint32_t cols, void* wt, hipStream_t s)
{
    const dim3 grid((cols + 63) / 64, (rows + 63) / 64);
    if (grid.y > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(transpose16_kernel, grid, dim3(kThreads), 0, s, static_cast<const uint16_t*>(w), rows, cols,
                       static_cast<uint16_t*>(wt));
    return hipGetLastError();
}

// y [M][out] = x [M][in] . wt [out][in]^T; scale (device, may be NULL) multiplies the finished sum; `partial` holds
// layer_gemm_partial_bytes(...) bytes
hipError_t launch_layer_gemm(const void* x, uint32_t M, const void* wt, int dtype, uint32_t in_features, uint32_t out_features,
                             const float* scale, const void* bias, void* y, float* partial, hipStream_t s)
{
    const GemmShape g = gemm_shape(M, in_features, out_features);
    const dim3 grid(8 * ((g.whole + 7) / 8) + 8 * ((g.jobs - g.whole + 7) / 8));
    const uint16_t* xs = static_cast<const uint16_t*>(x);
    const uint16_t* ws = static_cast<const uint16_t*>(wt);
    const uint16_t* bs = static_cast<const uint16_t*>(bias);
    uint16_t* ys = static_cast<uint16_t*>(y);
    if (dtype != 1 && dtype != 2) return hipErrorInvalidValue;
    static bool lds_set[3] = {};
    if (!lds_set[dtype]) {
        const void* fn = dtype == 1 ? reinterpret_cast<const void*>(&gemm_tn_kernel<1>) : reinterpret_cast<const void*>(&gemm_tn_kernel<2>);
        const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, int(kGemmLdsBytes));
        if (e != hipSuccess) return e;
        lds_set[dtype] = true;
    }
    if (dtype == 1)
        hipLaunchKernelGGL(gemm_tn_kernel<1>, grid, dim3(kThreads), kGemmLdsBytes, s, xs, ws, M, out_features, in_features, scale,
                           bs, ys, partial, g.m_tiles, g.whole, g.f, g.k_per_split, g.jobs);
    else
        hipLaunchKernelGGL(gemm_tn_kernel<2>, grid, dim3(kThreads), kGemmLdsBytes, s, xs, ws, M, out_features, in_features, scale,
                           bs, ys, partial, g.m_tiles, g.whole, g.f, g.k_per_split, g.jobs);
    if (g.cut_tiles > 0) {
        const dim3 fgrid(BM * BN / kThreads, g.cut_tiles);
        if (dtype == 1)
            hipLaunchKernelGGL(gemm_finish_kernel<1>, fgrid, dim3(kThreads), 0, s, partial, M, out_features, g.m_tiles, g.whole,
                               g.f, scale, bs, ys);
        else
            hipLaunchKernelGGL(gemm_finish_kernel<2>, fgrid, dim3(kThreads), 0, s, partial, M, out_features, g.m_tiles, g.whole,
                               g.f, scale, bs, ys);
    }
    return hipGetLastError();
}

}  // namespace cc
