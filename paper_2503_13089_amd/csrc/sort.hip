// Norm ordering for the pruned E-step (Section 3.1: the codes are the argmin over ALL centroids; a
// centroid can be skipped for a vector only if it provably cannot be that argmin).
//
// Triangle inequality: ||x - c|| >= | ||x|| - ||c|| |. If some centroid is known to lie within
// distance u of x (any centroid will do - the previous iteration's code is a good one), then every
// centroid with | ||c|| - ||x|| | > u is farther than that and cannot be the nearest. With the
// centroids ordered by norm this is a contiguous window of the codebook, and with the vectors ordered
// by norm too, the 512 vectors a workgroup scores share almost the same window.
//
// A second necessary condition comes from any fixed unit direction e: |e.c - e.x| <= ||c - x|| <= u.
// Both are folded into one 16-bit ordering key: 9 bits of norm shell (about 3 % wide, 511 shells below
// the largest possible norm, open-ended at both ends) and 7 bits of the cosine between the vector and
// e = (1,..,1)/sqrt(d). In that order the candidates of a vector are, per shell inside its norm band,
// one contiguous run of cosine buckets; the 512 neighbouring vectors a workgroup scores need almost
// the same runs.
//
// This file holds the ordering machinery: the keys, a stable two-pass LSD radix sort of (key, id)
// pairs whose output does not depend on scheduling, the row gather that builds the ordered copy of
// the vectors, the per-workgroup window lists, and the scatter of the codes back to input order.
#include <algorithm>

#include "common.h"

namespace cc {

constexpr int kThreads = 256;
constexpr int kSortThreads = 512;          // 8 waves
constexpr uint32_t kSortChunk = 4096;      // elements per block and pass

// 16-bit norm key: the top half of the fp32 pattern of a non-negative float (monotone, 2^-7 relative steps)
__device__ __forceinline__ uint32_t norm_key(float norm) { return __float_as_uint(norm) >> 16; }

// Shells: 4 norm keys each. `base` places shell 511 at the largest norm any vector can have; everything
// 511 shells (16 octaves) or more below that shares shell 0, anything above shares shell 511.
__device__ __forceinline__ uint32_t shell_base(uint32_t absmax_bits, int d)
{
    const float top = __uint_as_float(absmax_bits) * __builtin_sqrtf(float(d)) * 1.0001f;
    const uint32_t tk = norm_key(top) >> 2;
    return tk > 511u ? tk - 511u : 0u;
}
__device__ __forceinline__ uint32_t shell_of_key(uint32_t nkey, uint32_t base)
{
    const uint32_t s = nkey >> 2;
    return s <= base ? 0u : min(s - base, 511u);
}
// every norm whose key falls in shell s lies in [shell_rlo, shell_rhi)
__device__ __forceinline__ float shell_rlo(uint32_t s, uint32_t base)
{
    return s == 0 ? 0.0f : __uint_as_float(((s + base) << 2) << 16);
}
__device__ __forceinline__ float shell_rhi(uint32_t s, uint32_t base)
{
    return s >= 511u ? INFINITY : __uint_as_float(((s + base + 1) << 2) << 16);
}
__device__ __forceinline__ uint32_t cos_bucket(float t)
{
    const int q = int((t + 1.0f) * 64.0f);
    return uint32_t(max(0, min(q, 127)));
}
// norm, projection on e = (1,..,1)/sqrt(d), and the ordering key of one row
template <int D>
__device__ __forceinline__ uint32_t ordering_key(const float (&x)[D], float norm, uint32_t base, float& proj)
{
    float sum = 0.0f;
#pragma unroll
    for (int j = 0; j < D; ++j) sum += x[j];
    proj = sum * (D == 4 ? 0.5f : (D == 16 ? 0.25f : 0.35355339059327373f));
    const float t = norm > 0.0f ? proj / norm : 0.0f;
    return (shell_of_key(norm_key(norm), base) << 7) | cos_bucket(t);
}

template <int D>
__global__ __launch_bounds__(kThreads) void vector_keys_kernel(const float* __restrict__ X, uint32_t N,
                                                               uint16_t* __restrict__ keys, uint32_t* __restrict__ ids,
                                                               const WsHeader* __restrict__ hdr)
{
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= N) return;
    float x[D];
    load_row<D>(X + size_t(i) * D, x);
    float s = 0.0f, proj;
#pragma unroll
    for (int j = 0; j < D; ++j) s = __builtin_fmaf(x[j], x[j], s);
    keys[i] = uint16_t(ordering_key<D>(x, __builtin_sqrtf(s), shell_base(hdr->absmax_bits, D), proj));
    ids[i] = i;
}

// One radix pass over 8 bits of the key. hist is digit-major: hist[digit * blocks + block].
__global__ __launch_bounds__(kSortThreads) void radix_hist_kernel(const uint16_t* __restrict__ keys, uint32_t n,
                                                                  uint32_t chunk, int shift, uint32_t* __restrict__ hist)
{
    __shared__ uint32_t h[256];
    if (threadIdx.x < 256) h[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t lo = blockIdx.x * chunk, hi = min(lo + chunk, n);
    for (uint32_t i = lo + threadIdx.x; i < hi; i += kSortThreads) atomicAdd(&h[(keys[i] >> shift) & 255u], 1u);
    __syncthreads();
    if (threadIdx.x < 256) hist[threadIdx.x * gridDim.x + blockIdx.x] = h[threadIdx.x];
}

// Row scan of the digit-major histogram: block `digit` replaces hist[digit][0..blocks) by its exclusive
// prefix sum and writes the row total to totals[digit]. The scatter adds the prefix of the totals itself.
__global__ __launch_bounds__(1024) void radix_rowscan_kernel(uint32_t* __restrict__ hist, uint32_t blocks,
                                                             uint32_t* __restrict__ totals)
{
    __shared__ uint32_t part[1024];
    uint32_t* row = hist + size_t(blockIdx.x) * blocks;
    uint32_t carry = 0;
    for (uint32_t base = 0; base < blocks; base += 1024) {
        const uint32_t i = base + threadIdx.x;
        const uint32_t v = i < blocks ? row[i] : 0;
        part[threadIdx.x] = v;
        __syncthreads();
        for (uint32_t off = 1; off < 1024; off <<= 1) {  // Hillis-Steele inclusive scan
            const uint32_t t = threadIdx.x >= off ? part[threadIdx.x - off] : 0;
            __syncthreads();
            part[threadIdx.x] += t;
            __syncthreads();
        }
        if (i < blocks) row[i] = carry + part[threadIdx.x] - v;
        carry += part[1023];
        __syncthreads();
    }
    if (threadIdx.x == 0) totals[blockIdx.x] = carry;
}

// Stable scatter of one pass: an element goes to (start of its digit for this block, from the scanned
// histogram) + (number of earlier elements of this block with the same digit). "Earlier" is by
// position, so the result is the same whatever the scheduling.
__global__ __launch_bounds__(kSortThreads) void radix_scatter_kernel(const uint16_t* __restrict__ keys_in,
                                                                     const uint32_t* __restrict__ ids_in, uint32_t n,
                                                                     uint32_t chunk, int shift,
                                                                     const uint32_t* __restrict__ hist,
                                                                     const uint32_t* __restrict__ totals,
                                                                     uint16_t* __restrict__ keys_out,
                                                                     uint32_t* __restrict__ ids_out)
{
    constexpr int kWaves = kSortThreads / 64;
    __shared__ uint32_t base[256];            // next free slot per digit
    __shared__ uint32_t cnt[kWaves][256];     // per round: elements of each digit in each wave
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // start of (digit, this block) = sum of the totals of all smaller digits + this block's row prefix
    if (threadIdx.x < 256) cnt[0][threadIdx.x] = totals[threadIdx.x];
    __syncthreads();
    if (threadIdx.x < 256) {
        uint32_t before = 0;
        for (uint32_t dg = 0; dg < threadIdx.x; ++dg) before += cnt[0][dg];
        base[threadIdx.x] = before + hist[threadIdx.x * gridDim.x + blockIdx.x];
    }
    __syncthreads();
    const uint32_t lo = blockIdx.x * chunk, hi = min(lo + chunk, n);
    for (uint32_t r0 = lo; r0 < hi; r0 += kSortThreads) {
        for (int t = threadIdx.x; t < kWaves * 256; t += kSortThreads) (&cnt[0][0])[t] = 0;
        __syncthreads();
        const uint32_t i = r0 + threadIdx.x;
        const bool live = i < hi;
        const uint32_t key = live ? keys_in[i] : 0;
        const uint32_t id = live ? ids_in[i] : 0;
        const uint32_t digit = (key >> shift) & 255u;
        // lanes of this wave holding the same digit
        unsigned long long same = __ballot(live);
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const unsigned long long set = __ballot(live && ((digit >> b) & 1u));
            same &= ((digit >> b) & 1u) ? set : ~set;
        }
        const uint32_t below = __popcll(same & ((1ull << lane) - 1ull));
        if (live && below == 0) cnt[wave][digit] = uint32_t(__popcll(same));  // one writer per (wave, digit)
        __syncthreads();
        uint32_t pos = 0;
        if (live) {
            pos = base[digit] + below;
            for (int w = 0; w < wave; ++w) pos += cnt[w][digit];
        }
        __syncthreads();
        if (threadIdx.x < 256) {
            uint32_t t = 0;
            for (int w = 0; w < kWaves; ++w) t += cnt[w][threadIdx.x];
            base[threadIdx.x] += t;
        }
        if (live) {
            keys_out[pos] = uint16_t(key);
            ids_out[pos] = id;
        }
        __syncthreads();
    }
}

// out_row[p] = in_row[ids[p]]
template <int D>
__global__ __launch_bounds__(kThreads) void gather_rows_kernel(const float* __restrict__ in,
                                                               const uint32_t* __restrict__ ids, uint32_t n,
                                                               float* __restrict__ out)
{
    constexpr int Q = D / 4;
    const uint64_t t = uint64_t(blockIdx.x) * kThreads + threadIdx.x;
    if (t >= uint64_t(n) * Q) return;
    const uint32_t p = uint32_t(t / Q), q = uint32_t(t % Q);
    reinterpret_cast<float4*>(out)[t] = reinterpret_cast<const float4*>(in)[size_t(ids[p]) * Q + q];
}

template <int D>
__global__ __launch_bounds__(kThreads) void centroid_keys_kernel(const float* __restrict__ C, uint32_t K,
                                                                 uint16_t* __restrict__ keys, uint32_t* __restrict__ ids,
                                                                 const WsHeader* __restrict__ hdr)
{
    const uint32_t k = blockIdx.x * kThreads + threadIdx.x;
    if (k >= K) return;
    float c[D];
    load_row<D>(C + size_t(k) * D, c);
    float s = 0.0f, proj;
#pragma unroll
    for (int j = 0; j < D; ++j) s = __builtin_fmaf(c[j], c[j], s);
    keys[k] = uint16_t(ordering_key<D>(c, __builtin_sqrtf(s), shell_base(hdr->absmax_bits, D), proj));
    ids[k] = k;
}

// Window list of one 512-vector tile: the runs of the ordered codebook (in units of kWinQuad = 32
// positions, one operand tile) that can hold the nearest centroid of any of its vectors. For vector x with
// bound u (the distance to its hinted centroid, slightly enlarged), a candidate c has its norm within u of
// ||x|| and its projection e.c within u of e.x. The tile takes the hull of those bands over its 512
// (neighbouring, hence similar) vectors; per shell s inside the norm band the cosine e.c/||c|| is then
// confined to [t_lo, t_hi] computed from the shell's radius range, i.e. to a run of ordering keys
// (s, q_lo..q_hi). Rounding slack: both bands are widened by 1e-5 of the largest norm in play and every cosine
// bound by 1e-4. The fp32 norms, projections and quotients behind them - here and where the centroids' keys were
// made - are each within a few 1e-7 of that scale of their exact values, and u already carries a factor 1.001,
// so the slack is some fifty times what rounding can move a bound. Runs of neighbouring shells that touch are
// merged. If the band spans more than kWinSlots shells the list degrades to the single run of all keys
// inside the norm band.
// guess > 0 (no codes yet): u = guess * ||x|| instead, a window that proves nothing but is likely to hold a
// centroid close to x; the nearest centroid inside it then serves as the hint of the real pass.
// Layout per tile: entry 0 = (number of runs, their total length), entries 1.. = (first quad, end quad).
template <int D>
__global__ __launch_bounds__(kThreads) void window_kernel(const float* __restrict__ Xs, uint32_t N,
                                                          const float* __restrict__ C, uint32_t K,
                                                          const uint32_t* __restrict__ hint, const WsPersist* persist,
                                                          const uint32_t* __restrict__ ckey_starts, float guess,
                                                          const WsHeader* __restrict__ hdr, uint2* __restrict__ win)
{
    __shared__ float red[4][kThreads / 64];
    __shared__ uint2 runs[kWinSlots];
    const uint32_t quads = (K + kWinQuad - 1) / kWinQuad;
    uint2* out = win + size_t(blockIdx.x) * kWinStride;
    const bool guessing = guess > 0.0f;
    if (guessing && persist->hint_valid != 0) return;  // a hint exists: the pass these windows are for will not run
    const uint32_t base = shell_base(hdr->absmax_bits, D);
    // phase 1: hull over the tile's vectors of the norm band [||x|| - u, ||x|| + u] and of the projection band
    // [e.x - u, e.x + u] (the hull of a union of intervals contains the union, so this only ever adds candidates)
    float nlo = INFINITY, nhi = 0.0f, plo = INFINITY, phi = -INFINITY;
#pragma unroll
    for (int v = 0; v < int(kWinTile) / kThreads; ++v) {
        const uint32_t p = blockIdx.x * kWinTile + v * kThreads + threadIdx.x;
        if (p < N) {
            float x[D];
            load_row<D>(Xs + size_t(p) * D, x);
            float s = 0.0f, prj;
#pragma unroll
            for (int j = 0; j < D; ++j) s = __builtin_fmaf(x[j], x[j], s);
            const float nrm = __builtin_sqrtf(s);
            float u;
            if (guessing) {
                u = guess * nrm + 1e-30f;
            } else {
                float c[D];
                load_row<D>(C + size_t(min(hint[p], K - 1)) * D, c);
                u = __builtin_sqrtf(direct_sqdist<D>(x, c)) * 1.001f + 1e-30f;
            }
            (void)ordering_key<D>(x, nrm, base, prj);
            nlo = __builtin_fminf(nlo, nrm - u);
            nhi = __builtin_fmaxf(nhi, nrm + u);
            plo = __builtin_fminf(plo, prj - u);
            phi = __builtin_fmaxf(phi, prj + u);
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        nlo = __builtin_fminf(nlo, __shfl_xor(nlo, off, 64));
        nhi = __builtin_fmaxf(nhi, __shfl_xor(nhi, off, 64));
        plo = __builtin_fminf(plo, __shfl_xor(plo, off, 64));
        phi = __builtin_fmaxf(phi, __shfl_xor(phi, off, 64));
    }
    if ((threadIdx.x & 63) == 0) {
        red[0][threadIdx.x >> 6] = nlo;
        red[1][threadIdx.x >> 6] = nhi;
        red[2][threadIdx.x >> 6] = plo;
        red[3][threadIdx.x >> 6] = phi;
    }
    __syncthreads();
    for (int w = 0; w < kThreads / 64; ++w) {
        nlo = __builtin_fminf(nlo, red[0][w]);
        nhi = __builtin_fmaxf(nhi, red[1][w]);
        plo = __builtin_fminf(plo, red[2][w]);
        phi = __builtin_fmaxf(phi, red[3][w]);
    }
    // Both bands are widened by 1e-5 of the largest norm in play: the norms, projections and distances behind them
    // (sums of d fp32 products, a square root) are each within a few 1e-7 of that scale of their exact values, for
    // the vectors here and for the centroids' own keys alike, and u already carries a factor 1.001.
    const float slack = nhi < 3.0e38f ? 1e-5f * nhi : 0.0f;
    nlo -= slack;
    nhi += slack;
    plo -= slack;
    phi += slack;
    // shells of the norm band
    const uint32_t ka = nlo > 0.0f ? norm_key(nlo) : 0u;
    const uint32_t kb = nhi < 3.0e38f ? norm_key(nhi) : 0xffffu;
    const uint32_t smin = shell_of_key(ka, base);
    const uint32_t smax = shell_of_key(kb, base);
    const bool wide = smax - smin + 1 > uint32_t(kWinSlots);
    // phase 3: key runs -> position runs (the ordered keys are ascending), in quads
    const uint32_t nslots = wide ? 1 : smax - smin + 1;
    if (threadIdx.x < nslots) {
        uint32_t klo, khi;
        if (wide) {
            klo = smin << 7;
            khi = (smax << 7) | 127u;
        } else {
            // cosine e.c/||c|| of a candidate in shell s: e.c in [plo, phi], ||c|| in [rlo, rhi); 1e-4 of slack for
            // the two divisions (the centroid's own, when its key was made, and the one here: 1e-7 each)
            const uint32_t sh = smin + threadIdx.x;
            const float rlo = shell_rlo(sh, base), rhi = shell_rhi(sh, base);
            float tlo, thi;
            if (plo >= 0.0f) tlo = rhi < INFINITY ? plo / rhi : 0.0f; else tlo = rlo > 0.0f ? plo / rlo : -1.0f;
            if (phi >= 0.0f) thi = rlo > 0.0f ? phi / rlo : 1.0f; else thi = rhi < INFINITY ? phi / rhi : 0.0f;
            const uint32_t qa = cos_bucket(__builtin_fmaxf(tlo - 1e-4f, -1.0f));
            const uint32_t qb = cos_bucket(__builtin_fminf(thi + 1e-4f, 1.0f));
            klo = (sh << 7) | qa;
            khi = (sh << 7) | qb;
        }
        uint2 r = make_uint2(0, 0);
        if (klo <= khi) {
            const uint32_t first = ckey_starts[klo], end = ckey_starts[khi + 1];  // keys are ascending
            if (first < end) r = make_uint2(first / kWinQuad, (end + kWinQuad - 1) / kWinQuad);
        }
        runs[threadIdx.x] = r;
    }
    __syncthreads();
    // One thread merges the (at most kWinSlots) runs in LDS; the list then leaves with one store per thread. (Merging
    // straight into global memory and reading the list back for its total made this serial tail the longest part
    // of the kernel.)
    __shared__ uint2 merged[kWinSlots];
    __shared__ uint32_t merged_n, merged_total;
    if (threadIdx.x == 0) {
        uint32_t n = 0;
        uint2 last = make_uint2(0, 0);
        for (uint32_t t = 0; t < nslots; ++t) {
            const uint2 r = runs[t];
            if (r.x >= r.y) continue;
            // touches or overlaps the previous run, or starts in the stage where it ended (positions ascend with
            // the shell): merge, so that no stage - and no tracking group - is ever visited twice
            if (n > 0 && r.x / kStageTiles <= (last.y - 1) / kStageTiles) {
                last.y = max(last.y, r.y);
                merged[n - 1] = last;
            } else {
                last = r;
                merged[n++] = last;
            }
        }
        if (n == 0) {
            // With a hint this cannot happen (the hinted centroid itself lies inside its own runs); stay safe. A guessed
            // window may well be empty: any one tile will do then, every centroid gives a valid bound.
            n = 1;
            const uint32_t q = min(ckey_starts[smin << 7] / kWinQuad, quads - 1);
            merged[0] = guessing ? make_uint2(q, q + 1) : make_uint2(0, quads);
        }
        uint32_t total = 0;
        for (uint32_t r = 0; r < n; ++r) total += merged[r].y - merged[r].x;
        merged_n = n;
        merged_total = total;
    }
    __syncthreads();
    if (threadIdx.x < merged_n) out[1 + threadIdx.x] = merged[threadIdx.x];
    if (threadIdx.x == 0) out[0] = make_uint2(merged_n, merged_total);
}

// Sum of the window sizes of the last E-step (statistics only).
__global__ __launch_bounds__(1024) void window_stats_kernel(const uint2* __restrict__ win, uint32_t tiles, uint32_t K,
                                                            WsHeader* hdr, int only_without_hint)
{
    if (only_without_hint && !gate_open(hdr, kGateAlways | kGateNoHint)) return;
    __shared__ unsigned long long red[16];
    unsigned long long s = 0;
    for (uint32_t t = blockIdx.x * 1024 + threadIdx.x; t < tiles; t += gridDim.x * 1024) s += win[size_t(t) * kWinStride].y;
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 16; ++w) s += red[w];
        atomicAdd(&hdr->window_stages, s);
        if (blockIdx.x == 0)
            atomicAdd(&hdr->window_total, static_cast<unsigned long long>(tiles) * ((K + kWinQuad - 1) / kWinQuad));
    }
}

// Codes back to input order: idx[ids[p]] = idx_sorted[p]; also records that the sorted codes are a usable hint.
__global__ __launch_bounds__(kThreads) void unpermute_kernel(const uint32_t* __restrict__ idx_sorted,
                                                             const uint32_t* __restrict__ ids, uint32_t n,
                                                             uint32_t* __restrict__ idx, WsPersist* persist)
{
    const uint32_t p = blockIdx.x * kThreads + threadIdx.x;
    if (p == 0) persist->hint_valid = 1;
    if (p < n) idx[ids[p]] = idx_sorted[p];
}

// The hint survives between calls only for the same problem shape.
__global__ void persist_check_kernel(WsPersist* persist, uint32_t N, uint32_t d, uint32_t K, int drop_hint)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    constexpr unsigned long long kMagic = 0x636c7573636f6d70ull;  // "cluscomp"
    if (drop_hint || persist->magic != kMagic || persist->N != N || persist->d != d || persist->K != K) {
        persist->magic = kMagic;
        persist->N = N;
        persist->d = d;
        persist->K = K;
        persist->hint_valid = 0;
    }
}

// ---------------------------------------------------------------------------------------------------
// Elements per block and pass: a large array streams through 4096-element chunks (8 rounds of the scatter's
// ranking per block); a small one (the centroids, every iteration) is latency-bound, so it is spread over as many
// blocks as it has rounds.
static uint32_t sort_chunk(uint64_t n) { return n <= (1u << 18) ? uint32_t(kSortThreads) : kSortChunk; }

static void radix_sort16(uint16_t* keys_a, uint32_t* ids_a, uint16_t* keys_b, uint32_t* ids_b, uint32_t n,
                         uint32_t* hist, hipStream_t s)
{
    const uint32_t chunk = sort_chunk(n);
    const uint32_t blocks = (n + chunk - 1) / chunk;
    // pass 1: low byte a -> b; pass 2: high byte b -> a
    uint32_t* totals = hist + size_t(256) * blocks;
    hipLaunchKernelGGL(radix_hist_kernel, dim3(blocks), dim3(kSortThreads), 0, s, keys_a, n, chunk, 0, hist);
    hipLaunchKernelGGL(radix_rowscan_kernel, dim3(256), dim3(1024), 0, s, hist, blocks, totals);
    hipLaunchKernelGGL(radix_scatter_kernel, dim3(blocks), dim3(kSortThreads), 0, s, keys_a, ids_a, n, chunk, 0, hist, totals,
                       keys_b, ids_b);
    hipLaunchKernelGGL(radix_hist_kernel, dim3(blocks), dim3(kSortThreads), 0, s, keys_b, n, chunk, 8, hist);
    hipLaunchKernelGGL(radix_rowscan_kernel, dim3(256), dim3(1024), 0, s, hist, blocks, totals);
    hipLaunchKernelGGL(radix_scatter_kernel, dim3(blocks), dim3(kSortThreads), 0, s, keys_b, ids_b, n, chunk, 8, hist, totals,
                       keys_a, ids_a);
}

// The same stable two-pass sort for other callers: keys_a/ids_a in, sorted keys_a/ids_a out; keys_b/ids_b hold n
// entries each and hist sort_hist_bytes(n) bytes.
size_t sort_hist_bytes(uint64_t n) { return (size_t(n) / sort_chunk(n) + 3) * 256 * 4; }

hipError_t launch_sort_u16(uint16_t* keys_a, uint32_t* ids_a, uint16_t* keys_b, uint32_t* ids_b, uint32_t n, uint32_t* hist,
                           hipStream_t s)
{
    if (n == 0) return hipSuccess;
    radix_sort16(keys_a, ids_a, keys_b, ids_b, n, hist, s);
    return hipGetLastError();
}

template <int D>
static void sort_vectors_t(const float* X, uint32_t N, const Workspace& w, hipStream_t s)
{
    hipLaunchKernelGGL(vector_keys_kernel<D>, dim3((N + kThreads - 1) / kThreads), dim3(kThreads), 0, s, X, N, w.vkeys,
                       w.vperm, w.hdr);
    radix_sort16(w.vkeys, w.vperm, w.vkeys_tmp, w.vperm_tmp, N, w.sort_hist, s);
    const uint64_t pieces = uint64_t(N) * (D / 4);
    hipLaunchKernelGGL(gather_rows_kernel<D>, dim3(uint32_t((pieces + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, X,
                       w.vperm, N, w.xsorted);
}

hipError_t launch_sort_vectors(const float* X, uint32_t N, uint32_t d, uint32_t K, const Workspace& w, bool drop_hint,
                               hipStream_t s)
{
    hipLaunchKernelGGL(persist_check_kernel, dim3(1), dim3(64), 0, s, w.persist, N, d, K, drop_hint ? 1 : 0);
    switch (d) {
        case 4: sort_vectors_t<4>(X, N, w, s); break;
        case 8: sort_vectors_t<8>(X, N, w, s); break;
        case 16: sort_vectors_t<16>(X, N, w, s); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// What the E-step needs from the ordered centroids, in one launch: the key -> first position table (starts[v] for
// v = 0 .. 65536), the inverse permutation (cinv[cperm[p]] = p) and the ordered copy of the rows.
template <int D>
__global__ __launch_bounds__(kThreads) void centroid_tables_kernel(const uint16_t* __restrict__ sorted_keys,
                                                                   const uint32_t* __restrict__ perm, uint32_t K,
                                                                   const float* __restrict__ C, uint32_t* __restrict__ starts,
                                                                   uint32_t* __restrict__ inv, float* __restrict__ csorted)
{
    constexpr int Q = D / 4;
    const uint32_t t = blockIdx.x * kThreads + threadIdx.x;
    if (t <= 65536u) {
        uint32_t a = 0, b = K;
        while (a < b) {
            const uint32_t m = (a + b) / 2;
            if (sorted_keys[m] >= t) b = m; else a = m + 1;
        }
        starts[t] = a;
    }
    if (t < K) inv[perm[t]] = t;
    if (uint64_t(t) < uint64_t(K) * Q)
        reinterpret_cast<float4*>(csorted)[t] = reinterpret_cast<const float4*>(C)[size_t(perm[t / Q]) * Q + t % Q];
}

template <int D>
static void sort_centroids_t(const float* C, uint32_t K, const Workspace& w, hipStream_t s)
{
    hipLaunchKernelGGL(centroid_keys_kernel<D>, dim3((K + kThreads - 1) / kThreads), dim3(kThreads), 0, s, C, K, w.ckeys,
                       w.cperm, w.hdr);
    radix_sort16(w.ckeys, w.cperm, w.ckeys_tmp, w.cperm_tmp, K, w.sort_hist, s);
    const uint64_t pieces = uint64_t(K) * (D / 4);
    const uint32_t threads = uint32_t(std::max<uint64_t>(pieces, 65537));
    hipLaunchKernelGGL(centroid_tables_kernel<D>, dim3((threads + kThreads - 1) / kThreads), dim3(kThreads), 0, s, w.ckeys,
                       w.cperm, K, C, w.key_starts, w.cinv, w.csorted);
}

hipError_t launch_sort_centroids(const float* C, uint32_t d, uint32_t K, const Workspace& w, hipStream_t s)
{
    switch (d) {
        case 4: sort_centroids_t<4>(C, K, w, s); break;
        case 8: sort_centroids_t<8>(C, K, w, s); break;
        case 16: sort_centroids_t<16>(C, K, w, s); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int D>
static void windows_t(const float* C, uint32_t N, uint32_t K, const Workspace& w, float guess, hipStream_t s)
{
    hipLaunchKernelGGL(window_kernel<D>, dim3((N + kWinTile - 1) / kWinTile), dim3(kThreads), 0, s, w.xsorted, N, C, K, w.idx_sorted,
                       w.persist, w.key_starts, guess, w.hdr, w.windows);
    hipLaunchKernelGGL(window_stats_kernel, dim3(32), dim3(1024), 0, s, w.windows, (N + kWinTile - 1) / kWinTile, K, w.hdr,
                       guess > 0.0f ? 1 : 0);
}

// guess = 0: windows from the codes in w.idx_sorted (which must be valid codes of these vectors, however stale).
// guess > 0: no codes needed - windows of relative half-width `guess` around every vector's own norm and
// projection, for the bootstrap pass that produces the first codes; does nothing if the workspace holds a hint.
hipError_t launch_windows(const float* C, uint32_t N, uint32_t d, uint32_t K, const Workspace& w, float guess,
                          hipStream_t s)
{
    switch (d) {
        case 4: windows_t<4>(C, N, K, w, guess, s); break;
        case 8: windows_t<8>(C, N, K, w, guess, s); break;
        case 16: windows_t<16>(C, N, K, w, guess, s); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_unpermute(uint32_t N, uint32_t* idx, const Workspace& w, hipStream_t s)
{
    hipLaunchKernelGGL(unpermute_kernel, dim3((N + kThreads - 1) / kThreads), dim3(kThreads), 0, s, w.idx_sorted, w.vperm, N,
                       idx, w.persist);
    return hipGetLastError();
}

}  // namespace cc
