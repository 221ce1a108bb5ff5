// E-step on the matrix cores (Section 3.1: w_i goes to the centroid minimising ||w_i - c||^2).
//
// ||x - c||^2 = ||x||^2 + (||c||^2 - 2 x.c), and ||x||^2 does not affect the argmin, so the hot loop
// evaluates the score s(x, c) = ||c||^2 + sum_j c_j * (-2 x_j) for every (vector, centroid) pair:
// d fused multiply-adds on an accumulator preset to ||c||^2, which is exactly what the fp32 MFMA
// instruction v_mfma_f32_32x32x2_f32 computes when ||c||^2 is its C operand (k = 2 per instruction,
// d/2 chained instructions per 32 x 32 tile of pairs).
//
// Operand roles: centroids are the A rows, vectors the B columns, so each lane ends up with the 16
// scores of ONE vector (column lane%32) against 16 centroids; lanes l and l+32 share a vector.
// The vector ALUs then only have to fold those scores into a running minimum: v_min3_f32 folds
// two new scores per instruction. Tracking the argmin per score would cost several instructions per
// pair, so the loop tracks, per lane, only
//     best   = smallest score seen,          grp = the group of centroids it came from,
//     second = smallest score of any OTHER group
// at group granularity (one group = kGroupTiles tiles = 16*kGroupTiles centroids per lane).
//
// Epilogue, per vector: the winning group of each half-wave is re-evaluated in direct form
// (sum_j (x_j - c_j)^2, accurate to ~1e-6 relative of the distance itself) to get the index; the two
// halves are merged by direct-form distance. The fp32 score carries an absolute rounding error of
// up to E = 2^-24 ((2d+1) ||c||^2 + d ||x||^2), which is NOT small against the distance when the
// centroid is close (||x - c||^2 << ||x||^2). So a vector is only accepted if no other group came
// within the guard band `delta` >= E(winner) + E(true nearest) of the best score; otherwise it is
// appended to a refine list and re-decided over all K centroids in direct form by a second kernel.
// With ||c||^2 <= 2||x||^2 + 2 D for both the winner and the true nearest centroid (triangle
// inequality, D = the winner's distance), delta = 2 * 2^-24 * ((5d+2) ||x||^2 + (4d+2) D).
//
// The codebook is re-laid out once per call ("packed") so that every LDS read in the hot loop is a
// conflict-free wide read of exactly the MFMA operand a lane needs, with rows permuted such that
// lane-half h, accumulator register r of tile t is centroid 32 t + 16 h + r.
#include "common.h"

namespace cc {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;  // 4 waves, one per SIMD
constexpr float kUnit = 5.9604644775390625e-08f;  // 2^-24
constexpr float kGuardSafety = 1.5f;

// ---------------------------------------------------------------------------------------------
// Packed codebook: per 32-centroid tile, [64 lanes][KS] A-operand values, then 32 x ||c||^2.
// Rows past K are padded with c = 0 and ||c||^2 = +inf, which can never win.
template <int D>
__global__ __launch_bounds__(kThreads) void pack_codebook_kernel(const float* __restrict__ C, uint32_t K,
                                                                 uint32_t ntiles, float* __restrict__ packed,
                                                                 WsHeader* hdr, int gate,
                                                                 const uint32_t* __restrict__ cperm)
{
    constexpr uint32_t KS = D / 2, TF = 64 * KS + 32;
    if (!gate_open(hdr, gate)) return;
    const size_t o = size_t(blockIdx.x) * kThreads + threadIdx.x;
    if (o == 0) hdr->refine_count = 0;
    if (o >= size_t(ntiles) * TF) return;
    const uint32_t tile = uint32_t(o / TF), r = uint32_t(o % TF);
    float val;
    if (r < 64 * KS) {
        const uint32_t lane = r / KS, ks = r % KS, h = lane >> 5, m = lane & 31;
        // MFMA output row m lives in half (m/4)%2, register (m%4) + 4*(m/8): give it centroid 16*half + register
        const uint32_t pos = 32 * tile + 16 * ((m >> 2) & 1) + (m & 3) + 4 * (m >> 3);
        const uint32_t k = (cperm != nullptr && pos < K) ? cperm[pos] : pos;  // norm order when pruning
        val = pos < K ? C[size_t(k) * D + 2 * ks + h] : 0.0f;
    } else {
        const uint32_t pos = 32 * tile + (r - 64 * KS);
        const uint32_t k = (cperm != nullptr && pos < K) ? cperm[pos] : pos;
        if (pos < K) {
            double s = 0.0;
            for (int j = 0; j < D; ++j) {
                const double c = double(C[size_t(k) * D + j]);
                s += c * c;
            }
            val = float(s);  // one rounding
        } else {
            val = INFINITY;
        }
    }
    packed[o] = val;
}

// ---------------------------------------------------------------------------------------------
// WINDOWED = false: the whole packed codebook in stages of ST tiles. WINDOWED = true: the runs of the
// workgroup's window list (stages of kStageTiles tiles, tiles outside a run skipped).
template <int D, int VT, int ST, int GT, bool WINDOWED>
__global__ __launch_bounds__(kThreads, 2) void assign_mfma_kernel(const float* __restrict__ X, uint32_t N,
                                                               const float* __restrict__ C, uint32_t K,
                                                               const float* __restrict__ packed, uint32_t ntiles,
                                                               uint32_t* __restrict__ idx, float* __restrict__ dmin,
                                                               WsHeader* hdr, uint32_t* __restrict__ refine_list,
                                                               uint32_t refine_cap, int gate, long long* sums,
                                                               uint32_t* counts, const uint2* __restrict__ windows,
                                                               const uint32_t* __restrict__ cperm, int hint_only,
                                                               uint32_t* __restrict__ prev_out,
                                                               uint32_t* __restrict__ changed)
{
    constexpr int KS = D / 2;                 // MFMA k-steps per tile
    if (!gate_open(hdr, gate)) return;        // uniform over the grid
    constexpr int TF = 64 * KS + 32;          // floats per packed tile
    constexpr int STAGE_F4 = ST * TF / 4;     // float4 per LDS stage
    constexpr int NPF = (STAGE_F4 + kThreads - 1) / kThreads;
    static_assert(ST % GT == 0, "a tracking group must not straddle LDS stages");
    static_assert(!WINDOWED || ST == int(kStageTiles), "window runs never share a stage of kStageTiles tiles");
    __shared__ float4 lds[2][STAGE_F4];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int h = lane >> 5, n = lane & 31;
    // a windowed launch starts with the last tiles of the norm order, whose windows are the widest (as in the fp16 kernel)
    const uint32_t wg = WINDOWED ? gridDim.x - 1 - blockIdx.x : blockIdx.x;
    const uint32_t vbase = (wg * 4 + wave) * (32 * VT);

    // B operands: lane (n, h) supplies -2 * x_n[2 ks + h] for k-step ks
    float b[VT][KS];
#pragma unroll
    for (int vt = 0; vt < VT; ++vt) {
        const uint32_t i = min(vbase + vt * 32 + n, N - 1);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) b[vt][ks] = -2.0f * X[size_t(i) * D + 2 * ks + h];
    }
    float best[VT], second[VT];
    uint32_t grp[VT];
#pragma unroll
    for (int vt = 0; vt < VT; ++vt) {
        best[vt] = INFINITY;
        second[vt] = INFINITY;
        grp[vt] = 0;
    }

    // ntiles is a multiple of ST (padding rows carry ||c||^2 = +inf), so every stage is whole
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

        // prefetch the next stage into registers while this one is consumed
        float4 pf[NPF];
#pragma unroll
        for (int p = 0; p < NPF; ++p) {
            const uint32_t j = min(threadIdx.x + p * kThreads, uint32_t(STAGE_F4 - 1));
            pf[p] = P4[size_t(sn) * STAGE_F4 + j];
        }

        const float* L = reinterpret_cast<const float*>(lds[cur]);
#pragma unroll 1
        for (uint32_t tt = 0; tt < ST; tt += GT) {
            float m[VT];
#pragma unroll
            for (int vt = 0; vt < VT; ++vt) m[vt] = INFINITY;
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                if (WINDOWED && (tt + g < g_lo || tt + g >= g_hi)) continue;  // wave-uniform: tile outside the run
                const float* T = L + (tt + g) * TF;
                float a[KS];
                if constexpr (KS == 2) {
                    const float2 t = *reinterpret_cast<const float2*>(T + lane * 2);
                    a[0] = t.x; a[1] = t.y;
                } else {
#pragma unroll
                    for (int q = 0; q < KS / 4; ++q) {
                        const float4 t = *reinterpret_cast<const float4*>(T + lane * KS + 4 * q);
                        a[4 * q + 0] = t.x; a[4 * q + 1] = t.y; a[4 * q + 2] = t.z; a[4 * q + 3] = t.w;
                    }
                }
                f32x16 cn;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 t = *reinterpret_cast<const float4*>(T + 64 * KS + 16 * h + 4 * q);
                    cn[4 * q + 0] = t.x; cn[4 * q + 1] = t.y; cn[4 * q + 2] = t.z; cn[4 * q + 3] = t.w;
                }
#pragma unroll
                for (int vt = 0; vt < VT; ++vt) {
                    f32x16 acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[0], b[vt][0], cn, 0, 0, 0);
#pragma unroll
                    for (int ks = 1; ks < KS; ++ks)
                        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ks], b[vt][ks], acc, 0, 0, 0);
#pragma unroll
                    for (int q = 0; q < 8; ++q) m[vt] = __builtin_fminf(__builtin_fminf(m[vt], acc[2 * q]), acc[2 * q + 1]);
                }
            }
            const uint32_t gid = (s * ST + tt) / GT;
#pragma unroll
            for (int vt = 0; vt < VT; ++vt) {
                second[vt] = __builtin_amdgcn_fmed3f(best[vt], second[vt], m[vt]);
                grp[vt] = m[vt] < best[vt] ? gid : grp[vt];
                asm("v_min_f32 %0, %1, %2" : "=v"(best[vt]) : "v"(best[vt]), "v"(m[vt]));  // operands are canonical
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

    // ---- epilogue: index recovery in direct form, merge of the two half-waves, guard-band test
    const int sum_exp = sums != nullptr ? fixed_point_exp(hdr->absmax_bits, N) : 0;  // read once, not per vector
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
        float xn = 0.0f;
#pragma unroll
        for (int j = 0; j < D; ++j) xn = __builtin_fmaf(x[j], x[j], xn);
        const float delta = kGuardSafety * 2.0f * kUnit * (float(5 * D + 2) * xn + float(4 * D + 2) * dstar) + 1e-36f;
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
    constexpr int GT = int(kGroupTiles);
    constexpr uint32_t TF = 64 * (D / 2) + 32;
    const size_t packed_floats = size_t(e.packed_tiles) * TF;
    hipLaunchKernelGGL(pack_codebook_kernel<D>, dim3(uint32_t((packed_floats + kThreads - 1) / kThreads)),
                       dim3(kThreads), 0, s, e.pack_rows, e.K, e.packed_tiles, static_cast<float*>(e.packed), w.hdr, e.gate,
                       e.pack_perm);
    constexpr int VTW = VT * 128 > int(kWinTile) ? int(kWinTile) / 128 : VT;
    const uint32_t per_block = 4 * 32 * (e.windows != nullptr ? VTW : VT);
    const auto kernel = e.windows != nullptr ? assign_mfma_kernel<D, VTW, int(kStageTiles), GT, true>
                                             : assign_mfma_kernel<D, VT, ST, GT, false>;
    {
        ProfileScope scope(e.profile, kProfEstepF32, s);
        hipLaunchKernelGGL(kernel, dim3((e.N + per_block - 1) / per_block), dim3(kThreads), 0, s,
                           e.X, e.N, e.rows, e.K, static_cast<const float*>(e.packed), e.packed_tiles, e.idx, w.dmin, w.hdr,
                           w.refine_list, w.refine_cap, e.gate, e.accumulate ? w.sums : nullptr,
                           e.accumulate ? w.counts : nullptr, e.windows, e.row_ids, e.hint_only ? 1 : 0,
                           e.prev_out, e.changed);
    }
    return hipGetLastError();
}

hipError_t launch_assign_mfma_f32(const EStep& e, uint32_t d, const Workspace& w, hipStream_t s)
{
    switch (d) {
        case 4: return launch_t<4, 4, 8>(e, w, s);
        case 8: return launch_t<8, 4, 8>(e, w, s);
        case 16: return launch_t<16, 2, 4>(e, w, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace cc
