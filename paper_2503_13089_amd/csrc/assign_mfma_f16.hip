// E-step on the fp16 matrix cores with fp32-grade scores, for fp16-representable inputs
// (Section 3.1: w_i goes to the centroid minimising ||w_i - c||^2; the paper's tensors are 16-bit).
//
// Same scheme as the fp32 MFMA kernel (scores s = ||c||^2 - 2 x.c, lane = one vector, running
// min / second-min per centroid group, direct-form index recovery, guard band + refinement), but
// the products run on v_mfma_f32_32x32x16_f16, whose rate is 16x that of the fp32 MFMA and which,
// unlike the fp32 MFMA, leaves the vector ALUs free for the min-reduction while it runs.
//
// Exactness: every input x of the fp16 normal range is an fp16 number (checked on the device; otherwise the
// fp32 kernel runs); smaller ones may lose up to 2^-25 in the operand, which the guard band accounts for.
// Each fp32 centroid component, scaled by a power of two sigma so that it fits the fp16 range, is
// split into fp16 parts c*sigma = h1 + h2 (+ h3), each part the fp16 rounding of what is left. An
// fp16 x fp16 product has at most 22 significant bits, so every product h_p * (-2 x) is exact in the
// fp32 accumulator: the only rounding is in the accumulation. d = 4 takes three parts (residual below
// 2^-33 |c*sigma| or the fp16 subnormal step 2^-24): the k = 16 slots of one MFMA hold the 12 products
// and three more slots that add sigma * ||c||^2, itself split into three fp16 parts against the fixed
// multipliers 2^8, 2^-3, 2^-14. d = 8 and 16 take two parts (residual 2^-22 |c*sigma|, which the guard
// band carries as a term of its own - about a quarter on top of the accumulation term): 16 and 32
// slots, one and two MFMAs per tile instead of the two and three that three parts would need, with
// sigma * ||c||^2 as the fp32 C operand.
//
// Guard band: measured on gfx950, the accumulated result differs from the exact sum by at most
// ~3 * 2^-24 * (sum of |terms|), where the matrix core aligns a product by the exponent FIELDS of its
// factors: an fp16 subnormal factor counts as 2^-14 however small it is, so a nonzero product a * b
// weighs max(|a|, 2^-14) * max(|b|, 2^-14) in that sum (a subnormal norm part against the 2^8
// multiplier costs an absolute 2^-6 * 2^-24, for instance). The band assumes kAccumUlps = 8 times
// 2^-24 times that inflated sum, plus the split residual. A vector whose best and second-best group
// scores are closer than the band is re-decided in direct form over all K (refine.hip), exactly as
// for the fp32 kernel.
#include <algorithm>

#include "common.h"

namespace cc {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

constexpr int kThreads = 256;
constexpr float kUnit = 5.9604644775390625e-08f;  // 2^-24
constexpr float kGuardSafety = 1.5f;
constexpr float kAccumUlps = 8.0f;

template <int D>
struct F16Shape {
    static constexpr int kParts = (D == 4) ? 3 : 2;         // fp16 parts per centroid component
    static constexpr bool kNormInK = (D == 4);              // ||c||^2 rides in spare k slots
    static constexpr int kSlots = kParts * D + (kNormInK ? 3 : 0);
    static constexpr int KM = (kSlots + 15) / 16;           // MFMAs per tile
    static constexpr int kTileBytes = 64 * KM * 16 + (kNormInK ? 0 : 128);
};

// log2 of the centroid scale sigma: max|c| * sigma <= 2^15 and d * max|c|^2 * sigma <= 2^23
__device__ __forceinline__ int centroid_scale_log2(uint32_t cmax_bits, int d)
{
    if (cmax_bits == 0) return 0;
    const int ec = int(cmax_bits >> 23) - 127;  // max|c| < 2^(ec+1)
    const int ld = 32 - __clz(uint32_t(d - 1)); // d <= 2^ld
    int s = min(14 - ec, 21 - 2 * ec - ld);
    return max(-100, min(100, s));
}

// The three fp16 parts of a scaled fp32 value.
__device__ __forceinline__ void split3(float v, _Float16 (&h)[3])
{
    h[0] = _Float16(v);
    const float r1 = v - float(h[0]);  // exact
    h[1] = _Float16(r1);
    const float r2 = r1 - float(h[1]);  // exact
    h[2] = _Float16(r2);
}

// sigma*||c||^2 as g0*2^8 + g1*2^-3 + g2*2^-14
__device__ __forceinline__ void split_norm(float v, _Float16 (&g)[3])
{
    g[0] = _Float16(v * 0.00390625f);
    const float r1 = v - float(g[0]) * 256.0f;
    g[1] = _Float16(r1 * 8.0f);
    const float r2 = r1 - float(g[1]) * 0.125f;
    g[2] = _Float16(r2 * 16384.0f);
}

__global__ __launch_bounds__(kThreads) void codebook_absmax_kernel(const float4* __restrict__ C4, size_t n4,
                                                                   WsHeader* hdr, int gate)
{
    if (!gate_open(hdr, gate)) return;
    uint32_t m = 0;
    for (size_t i = size_t(blockIdx.x) * kThreads + threadIdx.x; i < n4; i += size_t(gridDim.x) * kThreads) {
        const float4 t = C4[i];
        m = max(max(m, __float_as_uint(t.x) & 0x7fffffffu), __float_as_uint(t.y) & 0x7fffffffu);
        m = max(max(m, __float_as_uint(t.z) & 0x7fffffffu), __float_as_uint(t.w) & 0x7fffffffu);
    }
    for (int off = 32; off > 0; off >>= 1) m = max(m, uint32_t(__shfl_xor(int(m), off, 64)));
    if ((threadIdx.x & 63) == 0 && m > __builtin_nontemporal_load(&hdr->cmax_bits)) atomicMax(&hdr->cmax_bits, m);
    if (blockIdx.x == 0 && threadIdx.x == 0) hdr->refine_count = 0;
}

// Packed codebook: per 32-centroid tile, [64 lanes][KM] x 8 fp16 A-operand values (lane (m, h) holds
// k slots 16*mi + 8h .. +7 of MFMA mi for output row m), then for d = 16 the 32 scaled norms (fp32).
// Output row m of a tile is centroid 32*tile + 16*((m/4)%2) + (m%4) + 4*(m/8), so that lane-half h,
// accumulator register r is centroid 32*tile + 16h + r. Rows past K: all-zero parts, norm = +inf.
template <int D>
__global__ __launch_bounds__(kThreads) void pack_codebook_f16_kernel(const float* __restrict__ C, uint32_t K,
                                                                     uint32_t ntiles, char* __restrict__ packed,
                                                                     const WsHeader* __restrict__ hdr, int gate,
                                                                     const uint32_t* __restrict__ cperm)
{
    using S = F16Shape<D>;
    if (!gate_open(hdr, gate)) return;
    const uint32_t t = blockIdx.x * kThreads + threadIdx.x;
    const uint32_t tile = t / 64, lane = t % 64;
    if (tile >= ntiles) return;
    const float sigma = __builtin_ldexpf(1.0f, centroid_scale_log2(hdr->cmax_bits, D));
    const uint32_t h = lane >> 5, m = lane & 31;
    const uint32_t pos = 32 * tile + 16 * ((m >> 2) & 1) + (m & 3) + 4 * (m >> 3);
    const bool valid = pos < K;
    const uint32_t k = (cperm != nullptr && valid) ? cperm[pos] : pos;  // norm order when pruning
    _Float16 parts[D][3];  // the first S::kParts are used
    double norm = 0.0;
#pragma unroll
    for (int j = 0; j < D; ++j) {
        const float c = valid ? C[size_t(k) * D + j] : 0.0f;
        norm += double(c) * double(c);
        split3(c * sigma, parts[j]);
    }
    _Float16 g[3];
    if (valid) {
        split_norm(float(norm * double(sigma)), g);  // one rounding of the exact norm
    } else {
        g[0] = _Float16(INFINITY);  // times the 2^8 multiplier: a score of +inf, never the minimum
        g[1] = _Float16(0.0f);
        g[2] = _Float16(0.0f);
    }
    char* tile_base = packed + size_t(tile) * S::kTileBytes;
#pragma unroll
    for (int mi = 0; mi < S::KM; ++mi) {
        f16x8 lo, hi;  // the slots of half 0 and of half 1
#pragma unroll
        for (int q8 = 0; q8 < 8; ++q8) {
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int q = 16 * mi + 8 * half + q8;
                _Float16 v = _Float16(0.0f);
                if (q < S::kParts * D) v = parts[q % D][q / D];
                else if (S::kNormInK && q < S::kParts * D + 3) v = g[q - S::kParts * D];
                if (half == 0) lo[q8] = v; else hi[q8] = v;
            }
        }
        *reinterpret_cast<f16x8*>(tile_base + (size_t(lane) * S::KM + mi) * 16) = h ? hi : lo;
    }
    if (!S::kNormInK && lane < 32) {
        // norms in centroid order 32*tile + lane (this thread's own k is a permuted row, so recompute)
        const uint32_t pc = 32 * tile + lane;
        const uint32_t kc = (cperm != nullptr && pc < K) ? cperm[pc] : pc;
        float v = INFINITY;
        if (pc < K) {
            double s = 0.0;
            for (int j = 0; j < D; ++j) {
                const double c = double(C[size_t(kc) * D + j]);
                s += c * c;
            }
            v = float(s * double(sigma));
        }
        *reinterpret_cast<float*>(tile_base + 64 * S::KM * 16 + 4 * lane) = v;
    }
}

// WINDOWED = false: the whole packed codebook in stages of ST tiles. WINDOWED = true: the runs of the
// workgroup's window list (stages of kStageTiles tiles, tiles outside a run skipped).
template <int D, int VT, int ST, int GT, bool WINDOWED>
__global__ __launch_bounds__(kThreads, 2) void assign_mfma_f16_kernel(
    const float* __restrict__ X, uint32_t N, const float* __restrict__ C, uint32_t K, const char* __restrict__ packed,
    uint32_t ntiles, uint32_t* __restrict__ idx, float* __restrict__ dmin, WsHeader* hdr,
    uint32_t* __restrict__ refine_list, uint32_t refine_cap, int gate,
    long long* sums, uint32_t* counts, const uint2* __restrict__ windows, const uint32_t* __restrict__ cperm, int hint_only,
    uint32_t* __restrict__ prev_out, uint32_t* __restrict__ changed)
{
    using S = F16Shape<D>;
    constexpr int KM = S::KM;
    constexpr int TILE_F4 = S::kTileBytes / 16;
    constexpr int STAGE_F4 = ST * TILE_F4;
    constexpr int NPF = (STAGE_F4 + kThreads - 1) / kThreads;
    static_assert(ST % GT == 0, "a tracking group must not straddle LDS stages");
    static_assert(!WINDOWED || ST == int(kStageTiles), "window runs never share a stage of kStageTiles tiles");
    if (!gate_open(hdr, gate)) return;  // uniform over the grid
    __shared__ float4 lds[2][STAGE_F4];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int h = lane >> 5, n = lane & 31;
    // A windowed launch starts with the last tiles of the norm order: the outer shells have the widest windows, and the
    // workgroups that take longest should not be the ones that start last (cfg3: 2.3 % of the fit; taking tiles from
    // both ends in turn instead costs 5 %).
    const uint32_t wg = WINDOWED ? gridDim.x - 1 - blockIdx.x : blockIdx.x;
    const uint32_t vbase = (wg * 4 + wave) * (32 * VT);

    // B operands: lane (n, h) supplies k slots 16*mi + 8h .. +7 of vector n: -2 x_j for the product
    // slots, the fixed multipliers for the norm slots, 0 for unused slots
    f16x8 b[VT][KM];
#pragma unroll
    for (int vt = 0; vt < VT; ++vt) {
        const uint32_t i = min(vbase + vt * 32 + n, N - 1);
        float x[D];
        load_row<D>(X + size_t(i) * D, x);
#pragma unroll
        for (int mi = 0; mi < KM; ++mi) {
#pragma unroll
            for (int q8 = 0; q8 < 8; ++q8) {
                _Float16 v[2];
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const int q = 16 * mi + 8 * half + q8;
                    v[half] = _Float16(0.0f);
                    constexpr int PD = S::kParts * D;
                    if (q < PD) v[half] = _Float16(-2.0f * x[q % D]);
                    else if (S::kNormInK && q == PD) v[half] = _Float16(256.0f);
                    else if (S::kNormInK && q == PD + 1) v[half] = _Float16(0.125f);
                    else if (S::kNormInK && q == PD + 2) v[half] = _Float16(6.103515625e-05f);  // 2^-14
                }
                b[vt][mi][q8] = h ? v[1] : v[0];
            }
        }
    }
    float best[VT], second[VT];
    uint32_t grp[VT];
#pragma unroll
    for (int vt = 0; vt < VT; ++vt) {
        best[vt] = INFINITY;
        second[vt] = INFINITY;
        grp[vt] = 0;
    }

    const float4* P4 = reinterpret_cast<const float4*>(packed);
    // Stages to score: the whole packed codebook, or the runs of this workgroup's 512-vector tile.
    const uint2* wl = WINDOWED ? windows + size_t((wg * (4 * 32 * VT)) / kWinTile) * kWinStride : nullptr;
    const uint32_t nruns = WINDOWED ? wl[0].x : 1u;
    uint32_t run = 0;
    uint2 cur_run = WINDOWED ? wl[1] : make_uint2(0, ntiles);  // [first tile, end tile)
    uint32_t s = cur_run.x / ST;
    int cur = 0;
#pragma unroll
    for (int p = 0; p < NPF; ++p) {
        const uint32_t j = threadIdx.x + p * kThreads;
        if (NPF * kThreads == STAGE_F4 || j < STAGE_F4) lds[0][j] = P4[size_t(s) * STAGE_F4 + j];
    }
    __syncthreads();

    while (true) {
        // the stage after this one: next in the run, or the first of the next run, or none
        uint32_t sn = s + 1, run_n = run;
        uint2 next_run = cur_run;
        if (sn * ST >= cur_run.y) {
            run_n = run + 1;
            if (WINDOWED && run_n < nruns) {
                next_run = wl[1 + run_n];
                sn = next_run.x / ST;
            }
        }
        // tiles of this stage that belong to the run
        const uint32_t g_lo = cur_run.x > s * ST ? cur_run.x - s * ST : 0u;
        const uint32_t g_hi = min(cur_run.y - s * ST, uint32_t(ST));
        const bool has_next = run_n < nruns;
        if (!has_next) sn = s;  // the last iteration re-reads its own stage; the copy is never used

        float4 pf[NPF];
#pragma unroll
        for (int p = 0; p < NPF; ++p) {
            const uint32_t j = min(threadIdx.x + p * kThreads, uint32_t(STAGE_F4 - 1));
            pf[p] = P4[size_t(sn) * STAGE_F4 + j];
        }

        const char* L = reinterpret_cast<const char*>(lds[cur]);
#pragma unroll 1
        for (uint32_t tt = 0; tt < ST; tt += GT) {
            float m[VT];
#pragma unroll
            for (int vt = 0; vt < VT; ++vt) m[vt] = INFINITY;
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                if (WINDOWED && (tt + g < g_lo || tt + g >= g_hi)) continue;  // wave-uniform: tile outside the run
                const char* T = L + (tt + g) * S::kTileBytes;
                f16x8 a[KM];
#pragma unroll
                for (int mi = 0; mi < KM; ++mi) a[mi] = *reinterpret_cast<const f16x8*>(T + (lane * KM + mi) * 16);
                f32x16 cn;
                if constexpr (S::kNormInK) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) cn[r] = 0.0f;
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float4 t = *reinterpret_cast<const float4*>(T + 64 * KM * 16 + (16 * h + 4 * q) * 4);
                        cn[4 * q + 0] = t.x; cn[4 * q + 1] = t.y; cn[4 * q + 2] = t.z; cn[4 * q + 3] = t.w;
                    }
                }
#pragma unroll
                for (int vt = 0; vt < VT; ++vt) {
                    f32x16 acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[0], b[vt][0], cn, 0, 0, 0);
#pragma unroll
                    for (int mi = 1; mi < KM; ++mi)
                        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[mi], b[vt][mi], acc, 0, 0, 0);
#pragma unroll
                    for (int q = 0; q < 8; ++q) m[vt] = __builtin_fminf(__builtin_fminf(m[vt], acc[2 * q]), acc[2 * q + 1]);
                }
            }
            const uint32_t gid = (s * ST + tt) / GT;
#pragma unroll
            for (int vt = 0; vt < VT; ++vt) {
                second[vt] = __builtin_amdgcn_fmed3f(best[vt], second[vt], m[vt]);
                grp[vt] = m[vt] < best[vt] ? gid : grp[vt];
                // plain v_min_f32: both operands come from v_min3/v_med3 results, which are already canonical,
                // so the canonicalising v_max the compiler would put in front of fminf is not needed
                asm("v_min_f32 %0, %1, %2" : "=v"(best[vt]) : "v"(best[vt]), "v"(m[vt]));
            }
        }

#pragma unroll
        for (int p = 0; p < NPF; ++p) {
            const uint32_t j = threadIdx.x + p * kThreads;
            if (NPF * kThreads == STAGE_F4 || j < STAGE_F4) lds[cur ^ 1][j] = pf[p];
        }
        __syncthreads();
        if (!has_next) break;
        s = sn;
        run = run_n;
        cur_run = next_run;
        cur ^= 1;
    }

    // ---- epilogue: index recovery in direct form, merge of the two half-waves, guard-band test.
    // Scores are in sigma-scaled units; the band is scaled to match.
    // read once: the header's cache line is the target of the refine-list atomics below, and a reload per vector
    // (which the compiler would emit, since those atomics may alias it) costs a trip to memory each time
    const uint32_t cmax_bits = hdr->cmax_bits;
    const float sigma = __builtin_ldexpf(1.0f, centroid_scale_log2(cmax_bits, D));
    const float sigma_cmax = sigma * __uint_as_float(cmax_bits);
    const int sum_exp = sums != nullptr ? fixed_point_exp(hdr->absmax_bits, N) : 0;
#pragma unroll
    for (int vt = 0; vt < VT; ++vt) {
        const uint32_t i_raw = vbase + vt * 32 + n;
        const uint32_t i = min(i_raw, N - 1);
        float x[D];
        load_row<D>(X + size_t(i) * D, x);
        // The overall best group sits in one of the two lanes that share this vector; both lanes split its
        // tiles. The other lane's best group, like every other group, only matters through `second`.
        static_assert(GT % 2 == 0, "the two lanes of a vector split the tiles of the winning group");
        const float ob = __shfl_xor(best[vt], 32, 64);
        const float os = __shfl_xor(second[vt], 32, 64);
        const uint32_t og = uint32_t(__shfl_xor(int(grp[vt]), 32, 64));
        const bool mine = best[vt] < ob || (best[vt] == ob && h == 0);
        const int wh = mine ? h : 1 - h;
        const uint32_t wgrp = mine ? grp[vt] : og;
        const float bstar = __builtin_fminf(best[vt], ob);
        const float sstar = __builtin_fminf(__builtin_fminf(second[vt], os), __builtin_fmaxf(best[vt], ob));
        float bd;
        uint32_t bk;
        recover_group<D, GT>(x, C, cperm, K, wgrp, wh, h * (GT / 2), (h + 1) * (GT / 2), bd, bk);
        const float od = __shfl_xor(bd, 32, 64);
        const uint32_t ok = uint32_t(__shfl_xor(int(bk), 32, 64));
        const bool take = od < bd || (od == bd && ok < bk);
        const float dstar = take ? od : bd;
        const uint32_t kstar = take ? ok : bk;
        if (hint_only) {  // bootstrap pass: the code is only an upper bound for the next pass's windows
            if (h == 0 && i_raw < N) idx[i] = kstar;
            continue;
        }
        float xn = 0.0f, x1 = 0.0f, xlost = 0.0f;
#pragma unroll
        for (int j = 0; j < D; ++j) {
            xn = __builtin_fmaf(x[j], x[j], xn);
            x1 += __builtin_fabsf(x[j]);
            // what the fp16 operand -2 x_j lost: nonzero only below the fp16 normal range, at most 2^-25, exact in fp32
            const float t = -2.0f * x[j];
            xlost += __builtin_fabsf(t - float(_Float16(t)));
        }
        // accumulation rounding of winner + true nearest (||c||^2 <= 2||x||^2 + 2D for both); what fp16
        // subnormal factors add to the sum of |terms| (with a = 2^-14: each of the P*D product slots at most
        // a |2 x_j| + a |part| + a^2, the parts of one centroid summing to <= 1.002 sigma ||c||_1, and the
        // norm slots at most 2^-6 + 2^-17 + 2^-28); then the split residuals: 2^-25 per component against
        // |2 x_j|, twice, and the norm residual
        constexpr float kA = 6.103515625e-05f;  // 2^-14
        constexpr int P = S::kParts;
        const float inflation = 2.0f * float(P) * kA * x1 + 1.002f * kA * sigma * __builtin_sqrtf(float(D) * (2.0f * xn + 2.0f * dstar)) +
                                float(P * D) * kA * kA + (S::kNormInK ? 0.015634f : 0.0f);
        // two parts leave a relative residual: |c sigma - h1 - h2| <= 2^-22 |c sigma| per component (each part is a
        // rounding to 11 bits), against |2 x_j|: at most 2^-21 sigma ||x|| ||c|| per score, for the best and for its
        // competitor (three parts leave 2^-33, which the accumulation term dwarfs)
        const float split_rel = P == 2 ? 9.5367431640625e-07f * sigma * __builtin_sqrtf(xn * (2.0f * xn + 2.0f * dstar)) : 0.0f;
        // a lost part of -2 x_j moves every score of this vector by at most |it| * sigma * max|c| * 1.002 (the
        // parts of a centroid component), the best and its competitor in opposite directions at worst
        const float operand_loss = 2.0f * 1.002f * sigma_cmax * xlost;
        const float delta = kGuardSafety * 2.0f * kAccumUlps * kUnit * (sigma * (5.0f * xn + 4.0f * dstar) + inflation) +
                            kGuardSafety * (2.0f * kUnit * x1 + 1e-11f + operand_loss + split_rel) + 1e-36f;
        const bool safe = (sstar - bstar) > delta;  // false for NaN as well
        bool moved = false;
        if (h == 0 && i_raw < N) {
            if (changed != nullptr) {
                // the code this vector had so far, kept wherever the M-step will have to look at it again: the
                // code differs, or the refinement may still change it
                const uint32_t old = idx[i];
                moved = old != kstar || !safe;
                if (moved) prev_out[i] = old;
            }
            idx[i] = kstar;
            dmin[i] = dstar;
            if (sums != nullptr) accumulate_vector<D>(x, kstar, sums, counts, sum_exp, +1);
            if (!safe) {
                const uint32_t pos = atomicAdd(&hdr->refine_count, 1u);
                if (pos < refine_cap) refine_list[pos] = i;
            }
        }
        if (changed != nullptr) {  // uniform over the wave; lanes 0..31 hold the 32 consecutive vectors of this tile
            const unsigned long long m = __ballot(moved);
            if (lane == 0 && vbase + vt * 32 < N) changed[(vbase + vt * 32) >> 5] = uint32_t(m);
        }
    }
}

template <int D, int VT, int ST>
static hipError_t launch_t(const EStep& e, const Workspace& w, hipStream_t s)
{
    // Tiles per tracking group: the epilogue re-evaluates the winning group in direct form, 8 * GT centroids per
    // lane. Over the whole codebook that is noise and a wide group keeps the hot loop lean; a windowed launch
    // scores only a few per cent of the codebook, the epilogue is then a third of the kernel, so groups are narrower.
    // From 32768 centroids on, 8-tile groups pay over the whole codebook (19.0 -> 18.75 ms at K = 65536, N = 11.3 M);
    // at K = 4096 the doubled epilogue would cost more than the loop saves.
    // At d = 8 and 16 a window still holds most of the codebook (the bands narrow like K^(-1/d)), the loop dominates again
    // and 4-tile groups pay (8192 x 28672, d = 8, K = 65536: 10 iterations in 531 instead of 545 ms).
    constexpr int GT = 4, GT_WIDE = ST >= 8 ? 8 : 4, GT_WINDOWED = D >= 8 ? 4 : 2;
    const size_t n4 = size_t(e.K) * D / 4;
    hipLaunchKernelGGL(codebook_absmax_kernel, dim3(uint32_t(std::min<size_t>((n4 + kThreads - 1) / kThreads, 64))),
                       dim3(kThreads), 0, s, reinterpret_cast<const float4*>(e.pack_rows), n4, w.hdr, e.gate);
    hipLaunchKernelGGL(pack_codebook_f16_kernel<D>, dim3((e.packed_tiles * 64 + kThreads - 1) / kThreads),
                       dim3(kThreads), 0, s, e.pack_rows, e.K, e.packed_tiles, static_cast<char*>(e.packed), w.hdr, e.gate,
                       e.pack_perm);
    // a windowed workgroup scores the vectors of one window list (or a part of them)
    constexpr int VTW = VT * 128 > int(kWinTile) ? int(kWinTile) / 128 : VT;
    const uint32_t per_block = 4 * 32 * (e.windows != nullptr ? VTW : VT);
    const auto kernel = e.windows != nullptr ? assign_mfma_f16_kernel<D, VTW, int(kStageTiles), GT_WINDOWED, true>
                        : (e.K >= 32768  ? assign_mfma_f16_kernel<D, VT, ST, GT_WIDE, false>
                                         : assign_mfma_f16_kernel<D, VT, ST, GT, false>);
    {
        ProfileScope scope(e.profile, kProfEstepF16, s);
        hipLaunchKernelGGL(kernel, dim3((e.N + per_block - 1) / per_block), dim3(kThreads),
                           0, s, e.X, e.N, e.rows, e.K, static_cast<const char*>(e.packed), e.packed_tiles, e.idx, w.dmin, w.hdr,
                           w.refine_list, w.refine_cap, e.gate, e.accumulate ? w.sums : nullptr,
                           e.accumulate ? w.counts : nullptr, e.windows, e.row_ids, e.hint_only ? 1 : 0,
                           e.prev_out, e.changed);
    }
    return hipGetLastError();
}

hipError_t launch_assign_mfma_f16(const EStep& e, uint32_t d, const Workspace& w, hipStream_t s)
{
    switch (d) {
        case 4: return launch_t<4, 4, 8>(e, w, s);
        case 8: return launch_t<8, 4, 4>(e, w, s);
        case 16: return launch_t<16, 4, 4>(e, w, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace cc
