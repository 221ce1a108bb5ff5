// Forward pass of the compressed linear layer at prefill-sized batches (the paper's layer listing: rebuild the
// weight from (codebook, codes), then y = x . W + bias), as two hand-written kernels:
//
//   1. layer_weight_frag_kernel: the listing's gather, written straight into the register layout of the matrix
//      cores' B operand. One fragment = 32 output columns x 16 in-features = 64 lanes x 8 consecutive k = 1 KB, lane
//      (n % 32) + 32 ((k % 16) / 8); fragments of one column block are contiguous along k. 64 x 64 tiles through LDS:
//      codes are read along a row of W, fragments leave in whole cache lines. Padding (columns past out_features,
//      in-features past the end of the last fragment) is written as zeros.
//   2. gemm_frag_kernel: y[M][N] = x[M][K] . W on v_mfma_f32_32x32x16_{bf16,f16}. A workgroup of 8 waves owns a
//      256 x 256 tile of y, each wave 128 x 64 of it (4 x 2 accumulator tiles of 32 x 32, in registers for the whole
//      contraction), and steps through K in slices of 32. Only x goes through LDS (double-buffered, rows padded to 40
//      halves so that the 16-byte fragment reads of 16 lanes fall on 16 different bank quads). The fragments of W
//      come from memory as they are: one fully coalesced 1 KB load per fragment, requested two slices ahead. Every
//      memory instruction of the loop sits between two matrix instructions.
//      Products of two 16-bit values are exact in fp32; the sum is fp32 in a fixed order; bias (and, for the
//      quantised codebook, the scale) are applied to the finished sum and y is rounded once.
//      Workgroups are numbered so that one XCD (they are dealt to the 8 XCDs in turn) works on neighbouring column
//      panels with all row panels of x: its L2 then holds the fragments it is using, and x comes once per XCD.
//      Tiles that do not fill a round of the chip's workgroup slots are cut along the contraction: fp32 partial
//      tiles go to the workspace and a second kernel adds them in a fixed order - the result never depends on
//      scheduling.
//
// Bound: the bf16 / fp16 matrix cores (2 M N K flop against 2.5 PFLOP/s). Measured at M = 2048, 4096 x 11008: the
// product takes 189 us = 0.98 PFLOP/s. The same loop with every memory instruction taken out (matrix instructions
// only) takes 130 us: under sustained matrix work the chip clocks near 1.7 GHz instead of 2.4, and the 344 tiles take
// 1.5 rounds on 256 compute units where 1.34 would do - that, not 2.5 PFLOP/s, is the ceiling of this tile schedule.
// The rebuild is bound by one codebook row lookup per code, a cache line fill each (58 us for 45 M weights), not by
// the 2 bytes it writes per weight.
#include <algorithm>

#include "common.h"

namespace cc {

namespace {

constexpr int kThreads = 256;               // rebuild and finishing kernels
constexpr int WN = 4;                       // waves along the columns of a tile (2 along its rows)
constexpr int kGemmThreads = 128 * WN;
constexpr int BM = 256, BN = 64 * WN, BK = 32;
constexpr int LDT = BK + 8;                 // halves per LDS row (20 words: the 16-byte reads of 16 lanes hit 16 bank quads)
constexpr int kStageHalves = BM * LDT;
constexpr uint32_t kGemmLdsBytes = 2 * kStageHalves * 2;   // 40,960 bytes
constexpr int kFragHalves = 512;            // one B operand: 32 columns x 16 in-features

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

// ---- 1. rebuild into B-operand fragments: column block nb = n / 32, in-feature block kb = k / 16, fragment
// (nb * KB + kb) with KB = ceil(in_features / 16) blocks per column block, lane (n % 32) + 32 ((k % 16) / 8), 8 halves
// Three steps per 64 x 64 tile: the tile's codes (64 rows of W, the code columns that touch the tile) go to LDS with
// reads along the rows of the code matrix; then a wave takes one code column and its 64 lanes the 64 rows, so that
// the elements they write into the transposed tile are neighbours in LDS (lanes along n would hit the same banks);
// then the tile leaves as 2 x 4 fragments, 64 lanes x 16 bytes each.
constexpr int kWtTile = 64;
constexpr int kWtMaxCols = kWtTile + 2;  // code columns touching a tile: at most 64 / g + 2 <= 66 for g >= 1
__global__ __launch_bounds__(kThreads) void layer_weight_frag_kernel(const uint16_t* __restrict__ codebook, uint32_t K, uint32_t g,
                                                                     const uint16_t* __restrict__ codes, uint32_t per_row,
                                                                     uint32_t in_features, uint32_t out_features,
                                                                     uint32_t NB, uint32_t KB, uint16_t* __restrict__ wf)
{
    constexpr int T = kWtTile, LT = T + 8;
    __shared__ __attribute__((aligned(16))) uint16_t tile[T * LT];  // [n][k]
    __shared__ uint16_t ctile[T * kWtMaxCols];                      // [k][code column]
    const uint32_t n_lo = blockIdx.x * T, k0 = blockIdx.y * T;
    const uint32_t cn_lo = n_lo / g;
    const uint32_t cn_hi = min((n_lo + T - 1) / g, per_row - 1);
    const uint32_t cpr = cn_hi - cn_lo + 1;  // code columns that touch this tile
    const uint32_t items = T * cpr;
    const bool edge = n_lo + T > out_features || k0 + T > in_features;
    if (edge)  // padding is stored too, as zeros
        for (uint32_t e = threadIdx.x; e < T * LT / 2; e += kThreads) reinterpret_cast<uint32_t*>(tile)[e] = 0u;
    for (uint32_t it = threadIdx.x; it < items; it += kThreads) {
        const uint32_t kr = it / cpr, c = it % cpr;
        const uint32_t k = min(k0 + kr, in_features - 1);
        ctile[kr * cpr + c] = codes[size_t(k) * per_row + cn_lo + c];
    }
    __syncthreads();
    const int n_end = int(min(uint32_t(T), out_features - n_lo));
    for (uint32_t it = threadIdx.x; it < items; it += kThreads) {
        const uint32_t c = it / T, kr = it % T;
        if (k0 + kr >= in_features) continue;
        const uint32_t code = min(uint32_t(ctile[kr * cpr + c]), K - 1);
        const uint16_t* row = codebook + size_t(code) * g;
        const int nbase = int((cn_lo + c) * g) - int(n_lo);
        if (g == 4) {
            const uint2 r = *reinterpret_cast<const uint2*>(row);
            const uint16_t e[4] = {uint16_t(r.x), uint16_t(r.x >> 16), uint16_t(r.y), uint16_t(r.y >> 16)};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int n = nbase + j;
                if (n >= 0 && n < n_end) tile[n * LT + kr] = e[j];
            }
        } else if (g == 8) {
            const uint4 r = *reinterpret_cast<const uint4*>(row);
            const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int n = nbase + j;
                if (n >= 0 && n < n_end) tile[n * LT + kr] = uint16_t(w[j >> 1] >> (16 * (j & 1)));
            }
        } else {
            for (uint32_t j = 0; j < g; ++j) {
                const int n = nbase + int(j);
                if (n >= 0 && n < n_end) tile[n * LT + kr] = row[j];
            }
        }
    }
    __syncthreads();
    // fragment q = 4 (column block within the tile) + (in-feature block within the tile): a wave writes one, 1 KB
    const uint32_t lane = threadIdx.x & 63, l32 = lane & 31, h = lane >> 5;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const uint32_t q = pass * 4 + threadIdx.x / 64;
        const uint32_t nb = n_lo / 32 + q / 4, kb = k0 / 16 + q % 4;
        if (nb < NB && kb < KB)
            *reinterpret_cast<uint4*>(wf + (size_t(nb) * KB + kb) * kFragHalves + lane * 8) =
                *reinterpret_cast<const uint4*>(&tile[((q / 4) * 32 + l32) * LT + (q % 4) * 16 + 8 * h]);
    }
}

// The integers of a quantised codebook (8 bits: signed bytes; 4 bits: two's-complement nibbles, element e in byte
// e / 2, low nibble first) as 16-bit floats, exact in both formats: the codebook the rebuild above gathers from when
// the product runs over the integers themselves.
template <int DT>
__global__ __launch_bounds__(kThreads) void codebook_integers16_kernel(const uint8_t* __restrict__ qbook, int bits, uint32_t n,
                                                                       uint16_t* __restrict__ out)
{
    const uint32_t e = blockIdx.x * kThreads + threadIdx.x;
    if (e >= n) return;
    int q;
    if (bits == 8) q = int(static_cast<int8_t>(qbook[e]));
    else q = int(((uint32_t(qbook[e >> 1]) >> (4 * (e & 1))) & 0xFu) ^ 8u) - 8;
    out[e] = from_f32<DT>(float(q));
}

// ---- 2. the product
// Jobs: the tiles of y in whole rounds of the chip's workgroup slots take the full contraction and write y themselves
// (`whole` of them); the tiles of the last, partial round are each cut into f in-feature slices, so that the round
// is short and full instead of long and half empty, and leave fp32 partial tiles for gemm_finish_kernel. The cut
// depends on the shape alone.
template <int DT>
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_frag_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ wf, uint32_t M, uint32_t N, uint32_t K, uint32_t NB, uint32_t KB,
    const float* __restrict__ scale, const uint16_t* __restrict__ bias, uint16_t* __restrict__ y, float* __restrict__ partial,
    uint32_t m_tiles, uint32_t whole, uint32_t f, uint32_t k_per_split, uint32_t jobs)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, h = lane >> 5, l32 = lane & 31;
    const int wm = wave & 1, wn = wave >> 1;

    // job of this workgroup: XCD q (= blockIdx % 8) takes the q-th contiguous share of the whole tiles and then the
    // q-th share of the slices of the cut tiles; within a share the row panels of x vary fastest, so neighbours
    // share a column panel of W
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

    // x: global -> registers -> LDS in 16-byte pieces, BK / 8 per row and slice; thread t takes piece t % PR of rows
    // t / PR + RP i. Rows past the edge are clamped (their results are never stored); a piece past k_end is read from
    // the last valid piece of its row instead and goes to LDS as zeros (K and k_per_split are multiples of 8).
    // W: this wave's two column blocks, fragments straight from memory; a block past the last one is clamped (its
    // columns are never stored), a fragment past the end of the contraction reads the last one (and is never used).
    //
    // The global loads of the main loop are written as instructions, with the waits on them placed by hand: the
    // compiler otherwise moves each request down to the slice that uses it, where its whole latency is exposed. The
    // memory counter retires loads in order, so a wait names how many younger requests may still be in flight. Every
    // slice issues the same six requests, past the end of the contraction too (clamped addresses, results unused),
    // which keeps those numbers the same for every slice.
    constexpr int PR = BK / 8, RP = kGemmThreads / PR, NA = BM / RP;
    static_assert(NA == 2, "the wait counts below assume two pieces of x per thread and slice");
    const uint32_t prow = threadIdx.x / PR, pk = (threadIdx.x % PR) * 8;
    const uint16_t* a_src[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) a_src[i] = x + size_t(min(m0 + prow + RP * i, M - 1)) * K;
    const uint16_t* b_src[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
        b_src[j] = wf + size_t(min(n0 / 32 + wn * 2 + j, NB - 1)) * KB * kFragHalves + lane * 8;
    auto request = [](u32x4& r, const uint16_t* p) { asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(r) : "v"(p)); };
    auto a_addr = [&](int i, uint32_t k0) { return a_src[i] + (k0 + pk < k_end ? k0 + pk : K - 8); };
    auto b_addr = [&](int j, uint32_t k) { return b_src[j] + size_t(min(k / 16, KB - 1)) * kFragHalves; };
#define CC_GEMM_ARRIVED(younger, r) asm volatile("s_waitcnt vmcnt(" #younger ")" : "+v"((r)[0]), "+v"((r)[1]))
    auto stash = [&](const u32x4 (&a)[NA], int buf, uint32_t k0) {
        const uint32_t keep = k0 + pk < k_end ? 0xffffffffu : 0u;
        uint16_t* As = lds + buf * kStageHalves;
#pragma unroll
        for (int i = 0; i < NA; ++i) *reinterpret_cast<u32x4*>(&As[(prow + RP * i) * LDT + pk]) = a[i] & keep;
    };
    const uint16_t* a_lds = lds + (wm * 128 + l32) * LDT + 8 * h;
    auto read_frag = [&](u32x4& a, int i, int buf, int kk) {
        a = *reinterpret_cast<const u32x4*>(a_lds + buf * kStageHalves + 32 * i * LDT + 16 * kk);
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // One slice of 32 in-features = two batches of 8 matrix instructions (16 in-features each) with the barrier
    // between them. Every memory instruction of the loop is issued between two matrix instructions, one at a time: a
    // wave that issues its requests in a burst waits at them until the memory pipeline has taken those of all eight
    // waves, and issues no matrix instruction meanwhile (measured: loop without matrix instructions 111 us, matrix
    // instructions alone 85 us, both with the requests in bursts 209 us - the sum). The x fragments of the second
    // batch are read from LDS during the first four instructions of the first batch, those of the next slice's first
    // batch during the first four of the second batch, after the barrier. Batch t takes its fragments of W from ring
    // slot t % 4. Slices come in pairs so that every slot and buffer index is a constant. Requests of slice s, in
    // order: during the second half of its first batch x of slice s + 2 (2), then W of the second batch of slice s + 1
    // (2); during the second half of its second batch W of the first batch of slice s + 2 (2). What it needs, and how
    // many younger requests are out by then: W of its first batch (asked for in slice s - 2: 6), x of slice s + 1 for
    // LDS (slice s - 1: 8, this slice's four included), W of its second batch (slice s - 1, after x: 6).
    // (The hand-over to LDS also runs after the last slice, where it moves zeros.)
    u32x4 a0[4], a1[4], bq[4][2], ar[2][NA];
#define CC_GEMM_STEP(stmt)                     \
    stmt;                                      \
    __builtin_amdgcn_sched_barrier(0)
#define CC_GEMM_SLICE(P, k0)                                                                   \
    do {                                                                                       \
        CC_GEMM_ARRIVED(6, bq[2 * (P)]);                                                       \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        CC_GEMM_STEP(acc[0][0] = mma<DT>(a0[0], bq[2 * (P)][0], acc[0][0]));                   \
        CC_GEMM_STEP(read_frag(a1[0], 0, P, 1));                                               \
        CC_GEMM_STEP(acc[0][1] = mma<DT>(a0[0], bq[2 * (P)][1], acc[0][1]));                   \
        CC_GEMM_STEP(read_frag(a1[1], 1, P, 1));                                               \
        CC_GEMM_STEP(acc[1][0] = mma<DT>(a0[1], bq[2 * (P)][0], acc[1][0]));                   \
        CC_GEMM_STEP(read_frag(a1[2], 2, P, 1));                                               \
        CC_GEMM_STEP(acc[1][1] = mma<DT>(a0[1], bq[2 * (P)][1], acc[1][1]));                   \
        CC_GEMM_STEP(read_frag(a1[3], 3, P, 1));                                               \
        CC_GEMM_STEP(acc[2][0] = mma<DT>(a0[2], bq[2 * (P)][0], acc[2][0]));                   \
        CC_GEMM_STEP(request(ar[P][0], a_addr(0, (k0) + 2 * BK)));                             \
        CC_GEMM_STEP(acc[2][1] = mma<DT>(a0[2], bq[2 * (P)][1], acc[2][1]));                   \
        CC_GEMM_STEP(request(ar[P][1], a_addr(1, (k0) + 2 * BK)));                             \
        CC_GEMM_STEP(acc[3][0] = mma<DT>(a0[3], bq[2 * (P)][0], acc[3][0]));                   \
        CC_GEMM_STEP(request(bq[(2 * (P) + 3) % 4][0], b_addr(0, (k0) + BK + 16)));            \
        CC_GEMM_STEP(acc[3][1] = mma<DT>(a0[3], bq[2 * (P)][1], acc[3][1]));                   \
        CC_GEMM_STEP(request(bq[(2 * (P) + 3) % 4][1], b_addr(1, (k0) + BK + 16)));            \
        CC_GEMM_ARRIVED(8, ar[1 - (P)]);                                                       \
        stash(ar[1 - (P)], 1 - (P), (k0) + BK);                                                \
        __syncthreads();                                                                       \
        CC_GEMM_ARRIVED(6, bq[2 * (P) + 1]);                                                   \
        __builtin_amdgcn_sched_barrier(0);                                                     \
        CC_GEMM_STEP(acc[0][0] = mma<DT>(a1[0], bq[2 * (P) + 1][0], acc[0][0]));               \
        CC_GEMM_STEP(read_frag(a0[0], 0, 1 - (P), 0));                                         \
        CC_GEMM_STEP(acc[0][1] = mma<DT>(a1[0], bq[2 * (P) + 1][1], acc[0][1]));               \
        CC_GEMM_STEP(read_frag(a0[1], 1, 1 - (P), 0));                                         \
        CC_GEMM_STEP(acc[1][0] = mma<DT>(a1[1], bq[2 * (P) + 1][0], acc[1][0]));               \
        CC_GEMM_STEP(read_frag(a0[2], 2, 1 - (P), 0));                                         \
        CC_GEMM_STEP(acc[1][1] = mma<DT>(a1[1], bq[2 * (P) + 1][1], acc[1][1]));               \
        CC_GEMM_STEP(read_frag(a0[3], 3, 1 - (P), 0));                                         \
        CC_GEMM_STEP(acc[2][0] = mma<DT>(a1[2], bq[2 * (P) + 1][0], acc[2][0]));               \
        CC_GEMM_STEP(acc[2][1] = mma<DT>(a1[2], bq[2 * (P) + 1][1], acc[2][1]));               \
        CC_GEMM_STEP(acc[3][0] = mma<DT>(a1[3], bq[2 * (P) + 1][0], acc[3][0]));               \
        CC_GEMM_STEP(request(bq[2 * (P)][0], b_addr(0, (k0) + 2 * BK)));                       \
        CC_GEMM_STEP(acc[3][1] = mma<DT>(a1[3], bq[2 * (P) + 1][1], acc[3][1]));               \
        CC_GEMM_STEP(request(bq[2 * (P)][1], b_addr(1, (k0) + 2 * BK)));                       \
    } while (0)

    // before the first slice: the same requests in the same order, as far as they exist
    request(ar[0][0], a_addr(0, k_begin));
    request(ar[0][1], a_addr(1, k_begin));
    request(bq[0][0], b_addr(0, k_begin));
    request(bq[0][1], b_addr(1, k_begin));
    request(ar[1][0], a_addr(0, k_begin + BK));
    request(ar[1][1], a_addr(1, k_begin + BK));
    request(bq[1][0], b_addr(0, k_begin + 16));
    request(bq[1][1], b_addr(1, k_begin + 16));
    request(bq[2][0], b_addr(0, k_begin + BK));
    request(bq[2][1], b_addr(1, k_begin + BK));
    CC_GEMM_ARRIVED(8, ar[0]);
    stash(ar[0], 0, k_begin);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) read_frag(a0[i], i, 0, 0);
    for (uint32_t k0 = k_begin;;) {
        CC_GEMM_SLICE(0, k0);
        if ((k0 += BK) >= k_end) break;
        CC_GEMM_SLICE(1, k0);
        if ((k0 += BK) >= k_end) break;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // requests past the end still write registers: let them land
#undef CC_GEMM_SLICE
#undef CC_GEMM_STEP
#undef CC_GEMM_ARRIVED

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

// Workgroups the chip holds at once: 256 compute units, each with room (registers) for the 8 waves of one workgroup.
constexpr uint32_t kGemmSlots = 256;

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

// bytes of the weight in fragment layout (whole fragments: columns padded to 32, in-features to 16)
size_t layer_weight_frag_bytes(uint32_t in_features, uint32_t out_features)
{
    return align256(size_t((out_features + 31) / 32) * ((in_features + 15) / 16) * kFragHalves * 2);
}

hipError_t launch_layer_weight_frag(const void* codebook, uint32_t K, uint32_t g, const uint16_t* codes, uint32_t in_features,
                                    uint32_t out_features, void* wf, hipStream_t s)
{
    const uint32_t per_row = (out_features + g - 1) / g;
    const dim3 grid((out_features + 63) / 64, (in_features + 63) / 64);
    if (grid.y > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(layer_weight_frag_kernel, grid, dim3(kThreads), 0, s, static_cast<const uint16_t*>(codebook), K, g, codes,
                       per_row, in_features, out_features, (out_features + 31) / 32, (in_features + 15) / 16,
                       static_cast<uint16_t*>(wf));
    return hipGetLastError();
}

hipError_t launch_codebook_integers16(const void* qbook, int bits, uint32_t K, uint32_t g, int dtype, void* book16, hipStream_t s)
{
    const uint32_t n = K * g;
    const dim3 grid((n + kThreads - 1) / kThreads);
    if (dtype == 1)
        hipLaunchKernelGGL(codebook_integers16_kernel<1>, grid, dim3(kThreads), 0, s, static_cast<const uint8_t*>(qbook), bits, n,
                           static_cast<uint16_t*>(book16));
    else if (dtype == 2)
        hipLaunchKernelGGL(codebook_integers16_kernel<2>, grid, dim3(kThreads), 0, s, static_cast<const uint8_t*>(qbook), bits, n,
                           static_cast<uint16_t*>(book16));
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

// y [M][out] = x [M][in] . W, W as written by launch_layer_weight_frag; scale (device, may be NULL) multiplies the
// finished sum; `partial` holds layer_gemm_partial_bytes(...) bytes
hipError_t launch_layer_gemm(const void* x, uint32_t M, const void* wf, int dtype, uint32_t in_features, uint32_t out_features,
                             const float* scale, const void* bias, void* y, float* partial, hipStream_t s)
{
    const GemmShape g = gemm_shape(M, in_features, out_features);
    const dim3 grid(8 * ((g.whole + 7) / 8) + 8 * ((g.jobs - g.whole + 7) / 8));
    const uint16_t* xs = static_cast<const uint16_t*>(x);
    const uint16_t* ws = static_cast<const uint16_t*>(wf);
    const uint16_t* bs = static_cast<const uint16_t*>(bias);
    uint16_t* ys = static_cast<uint16_t*>(y);
    const uint32_t NB = (out_features + 31) / 32, KB = (in_features + 15) / 16;
    if (dtype != 1 && dtype != 2) return hipErrorInvalidValue;
    if (dtype == 1)
        hipLaunchKernelGGL(gemm_frag_kernel<1>, grid, dim3(kGemmThreads), kGemmLdsBytes, s, xs, ws, M, out_features, in_features, NB,
                           KB, scale, bs, ys, partial, g.m_tiles, g.whole, g.f, g.k_per_split, g.jobs);
    else
        hipLaunchKernelGGL(gemm_frag_kernel<2>, grid, dim3(kGemmThreads), kGemmLdsBytes, s, xs, ws, M, out_features, in_features, NB,
                           KB, scale, bs, ys, partial, g.m_tiles, g.whole, g.f, g.k_per_split, g.jobs);
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
