// M-step by buckets (Section 3.1: c_k <- mean of the vectors assigned to cluster k), for K <= 65536.
//
// Summing straight into K accumulators needs one memory-side atomic per vector component, and those run
// at ~23 G/s on this chip: 2.4 ms for 11 M vectors of d = 4. Instead the vectors are first moved next to
// the other members of their bucket of 64 consecutive clusters, and one workgroup per bucket then adds
// its members up in LDS:
//   1. count:   per block of 4096 vectors, an LDS histogram of the buckets (one row of a blocks x buckets matrix),
//   2. scan:    two-level column scan of that matrix, prefix of the bucket totals = first record of every bucket,
//   3. scatter: every vector is copied, with its code, into a record of its bucket's range,
//   4. sum:     workgroup b adds the records of bucket b into 64 x (d sums + count) LDS accumulators
//               and writes the 64 means (an empty cluster keeps its previous centroid).
// The sums are the same 64-bit fixed-point integers as in the atomic formulation, so the order in which
// records land inside a bucket - the only thing here that depends on scheduling - cannot change a bit
// of the result.
//
// Because the sums are integers they can also be kept up to date instead of recomputed: inside a fit, from
// the third iteration on, only the vectors whose code changed since the previous iteration go through the
// four steps (18 % of them in the second iteration of the 4-bit benchmark, 2 % in the twentieth), each as
// two records - plus for the new cluster, minus for the old one - and step 4 adds the bucket's net change
// to the sums and counts that the previous iteration left in the workspace. Bit-identical to a recomputation.
// The E-step kernel that produced the codes leaves a bitmap of the vectors that may have changed (and their
// previous code), so steps 1 and 3 read one bit per vector instead of two code arrays.
#include <algorithm>

#include "common.h"

namespace cc {

constexpr int kThreads = 256;

// Exclusive prefix sum over the workgroup of one value per thread; `total` receives the sum.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* wave_sum, uint32_t& total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = v;
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = uint32_t(__shfl_up(int(incl), off, 64));
        if (lane >= off) incl += t;
    }
    __syncthreads();  // wave_sum may still be read from an earlier call
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    uint32_t before = incl - v;
    total = 0;
    for (int w = 0; w < kThreads / 64; ++w) {
        if (w < wave) before += wave_sum[w];
        total += wave_sum[w];
    }
    return before;
}

// The bucket of a code: by cluster index, or - with `cinv` (position of each centroid in the norm order of
// the E-step that produced the codes) - by that position, which neighbouring vectors of the ordered copy
// share, so that their records land next to each other.
__device__ __forceinline__ uint32_t slot_of_code(uint32_t k, const uint32_t* __restrict__ cinv)
{
    return cinv != nullptr ? cinv[k] : k;
}

// Calls f(i) for every flagged vector of the chunk of kDeltaChunk vectors starting at lo (bits beyond N are never
// set). Each thread reads the 64 flags of its own stretch (two words of the `changed` bitmap), the flagged offsets
// are packed into `list` (LDS, kDeltaChunk entries) and then dealt out evenly: with a few per cent of the flags set,
// a thread working through its own stretch alone would wait for the unluckiest lane of its wave.
template <typename F>
__device__ __forceinline__ void for_each_flagged(const uint32_t* __restrict__ changed, uint32_t lo, uint32_t N,
                                                 uint16_t* list, uint32_t* wave_sum, F f)
{
    static_assert(kDeltaChunk == 64 * kThreads && kDeltaChunk <= 65536, "two bitmap words per thread, 16-bit offsets");
    const uint32_t first = lo + 64 * threadIdx.x;
    uint32_t word[2] = {0u, 0u};
#pragma unroll
    for (uint32_t w = 0; w < 2; ++w)
        if (first + 32 * w < N) word[w] = changed[(first >> 5) + w];
    uint32_t total;
    uint32_t pos = block_exclusive_scan(uint32_t(__popc(word[0]) + __popc(word[1])), wave_sum, total);
#pragma unroll
    for (uint32_t w = 0; w < 2; ++w)
        for (uint32_t bits = word[w]; bits != 0; bits &= bits - 1)
            list[pos++] = uint16_t(64 * threadIdx.x + 32 * w + uint32_t(__ffs(int(bits)) - 1));
    __syncthreads();
    for (uint32_t e = threadIdx.x; e < total; e += kThreads) f(lo + list[e]);
}

// Which chunk of vectors a workgroup takes. Workgroups are dealt to the 8 XCDs in turn, and the records of
// neighbouring chunks are neighbours in every bucket's range: with chunk = workgroup id, each cache line on the
// border of two runs would be written in part by two XCDs, i.e. from two L2s that cannot merge the halves.
// This order gives each XCD a contiguous range of chunks instead (any bijection is correct; the histogram
// and the scatter pass only have to agree).
__device__ __forceinline__ uint32_t chunk_of_workgroup()
{
    const uint32_t n = gridDim.x, q = n / 8, r = n % 8, x = blockIdx.x % 8;
    return x * q + min(x, r) + blockIdx.x / 8;
}

// ---- 1. bucket histogram of one block of vectors: row `block` of hist[blocks][nbuckets]
__global__ __launch_bounds__(kThreads) void bucket_count_kernel(const uint32_t* __restrict__ idx,
                                                                const uint32_t* __restrict__ prev,
                                                                const uint32_t* __restrict__ changed, uint32_t N, uint32_t K,
                                                                const uint32_t* __restrict__ cinv, uint32_t nbuckets,
                                                                uint32_t* __restrict__ hist, WsHeader* hdr)
{
    __shared__ uint32_t h[kMaxBuckets];
    __shared__ uint32_t bad_total;
    __shared__ uint16_t flagged[kDeltaChunk];
    __shared__ uint32_t wave_sum[kThreads / 64];
    for (uint32_t b = threadIdx.x; b < nbuckets; b += kThreads) h[b] = 0;
    if (threadIdx.x == 0) bad_total = 0;
    __syncthreads();
    // a full pass works on chunks of kBucketChunk vectors; an incremental one (changed != NULL) on chunks of
    // kDeltaChunk, looks only at the flagged vectors, and counts one record for the new cluster and one for the old
    const uint32_t chunk = changed != nullptr ? kDeltaChunk : kBucketChunk;
    const uint32_t blk = chunk_of_workgroup();
    const uint32_t lo = blk * chunk, hi = min(lo + chunk, N);
    uint32_t bad = 0;
    if (changed != nullptr) {
        for_each_flagged(changed, lo, N, flagged, wave_sum, [&](uint32_t i) {
            const uint32_t k = idx[i], kp = prev[i];
            if (k != kp && k < K && kp < K) {
                atomicAdd(&h[slot_of_code(k, cinv) / kBucketClusters], 1u);
                atomicAdd(&h[slot_of_code(kp, cinv) / kBucketClusters], 1u);
            }
        });
    }
    for (uint32_t i = lo + threadIdx.x; changed == nullptr && i < hi; i += kThreads) {
        const uint32_t k = idx[i];
        if (k < K) atomicAdd(&h[slot_of_code(k, cinv) / kBucketClusters], 1u);
        else ++bad;
    }
    if (bad) atomicAdd(&bad_total, bad);
    __syncthreads();
    for (uint32_t b = threadIdx.x; b < nbuckets; b += kThreads) hist[size_t(blk) * nbuckets + b] = h[b];
    if (threadIdx.x == 0 && bad_total) atomicAdd(&hdr->skipped_vectors, static_cast<unsigned long long>(bad_total));
}

// ---- 2a. column scan, first level: within each group of kBucketGroup blocks, every column (bucket) of hist
// becomes its exclusive prefix over the group's blocks; the group's column sums go to gtot[group][bucket].
// One thread per (group, bucket); neighbouring threads read neighbouring buckets.
__global__ __launch_bounds__(kThreads) void bucket_groupscan_kernel(uint32_t* __restrict__ hist, uint32_t blocks,
                                                                    uint32_t nbuckets, uint32_t* __restrict__ gtot)
{
    const uint32_t b = blockIdx.x * kThreads + threadIdx.x;
    if (b >= nbuckets) return;
    const uint32_t first = blockIdx.y * kBucketGroup, last = min(first + kBucketGroup, blocks);
    uint32_t run = 0;
#pragma unroll 16
    for (uint32_t blk = first; blk < last; ++blk) {
        const size_t o = size_t(blk) * nbuckets + b;
        const uint32_t v = hist[o];
        hist[o] = run;
        run += v;
    }
    gtot[size_t(blockIdx.y) * nbuckets + b] = run;
}

// ---- 2b. second level, one workgroup: every column of gtot becomes its exclusive prefix over the groups, and the
// exclusive prefix of the column totals is the first record of every bucket (base[nbuckets] = number of records)
__global__ __launch_bounds__(kMaxBuckets) void bucket_base_kernel(uint32_t* __restrict__ gtot, uint32_t groups,
                                                                   uint32_t nbuckets, uint32_t* __restrict__ base)
{
    __shared__ uint32_t wave_sum[kMaxBuckets / 64];
    const uint32_t b = threadIdx.x;
    uint32_t run = 0;
    if (b < nbuckets) {
#pragma unroll 16
        for (uint32_t g = 0; g < groups; ++g) {
            const size_t o = size_t(g) * nbuckets + b;
            const uint32_t v = gtot[o];
            gtot[o] = run;
            run += v;
        }
    }
    // exclusive scan of `run` over the workgroup (one bucket per thread)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = run;
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = uint32_t(__shfl_up(int(incl), off, 64));
        if (lane >= off) incl += t;
    }
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    uint32_t before = incl - run, total = 0;
    for (int w = 0; w < int(kMaxBuckets / 64); ++w) {
        if (w < wave) before += wave_sum[w];
        total += wave_sum[w];
    }
    if (b < nbuckets) base[b] = before;
    if (b == 0) base[nbuckets] = total;
}

// A record: the d floats of the vector, then 16 bytes whose first word is the code's slot.
template <int D>
struct Record {
    static constexpr int kBytes = D * 4 + 16;
};

// ---- 3. copy every vector into its bucket's range. The block first orders its (vector, record position)
// pairs by bucket in LDS, then writes the records in that order, so that the records of one bucket leave
// as one contiguous run (isolated 32-byte writes reach only a fraction of the streaming bandwidth).
template <int D>
__global__ __launch_bounds__(kThreads) void bucket_scatter_kernel(const float* __restrict__ X, uint32_t N,
                                                                  const uint32_t* __restrict__ idx, uint32_t K,
                                                                  const uint32_t* __restrict__ cinv, uint32_t nbuckets,
                                                                  const uint32_t* __restrict__ hist,
                                                                  const uint32_t* __restrict__ gtot,
                                                                  const uint32_t* __restrict__ base,
                                                                  char* __restrict__ records)
{
    constexpr int kPer = kBucketChunk / kThreads;  // vectors per thread
    static_assert(kBucketChunk <= 8192 && kMaxBuckets * kBucketClusters <= (1u << 19), "packing of the stage entries");
    __shared__ uint32_t h[kMaxBuckets];            // members of each bucket in this block, then their first stage slot
    __shared__ uint32_t first_rec[kMaxBuckets];    // first record of (bucket, this block)
    __shared__ uint2 stage[kBucketChunk];          // (vector, record) in bucket order
    __shared__ uint32_t wave_sum[kThreads / 64];
    const uint32_t blk = chunk_of_workgroup();
    for (uint32_t b = threadIdx.x; b < nbuckets; b += kThreads) {
        h[b] = 0;
        first_rec[b] = base[b] + gtot[size_t(blk / kBucketGroup) * nbuckets + b] + hist[size_t(blk) * nbuckets + b];
    }
    __syncthreads();
    const uint32_t lo = blk * kBucketChunk;
    uint32_t slot[kPer], rank[kPer];
#pragma unroll
    for (int r = 0; r < kPer; ++r) {
        const uint32_t i = lo + r * kThreads + threadIdx.x;
        const uint32_t k = i < N ? idx[i] : 0xffffffffu;
        slot[r] = 0xffffffffu;
        rank[r] = 0;
        if (k < K) {  // codes >= K were counted by the histogram pass and are left out
            slot[r] = slot_of_code(k, cinv);
            rank[r] = atomicAdd(&h[slot[r] / kBucketClusters], 1u);
        }
    }
    __syncthreads();
    // exclusive prefix of h over the buckets: contiguous entries per thread, then the workgroup scan
    {
        const uint32_t per = (nbuckets + kThreads - 1) / kThreads;
        const uint32_t first = min(threadIdx.x * per, nbuckets), last = min(first + per, nbuckets);
        uint32_t s = 0;
        for (uint32_t b = first; b < last; ++b) s += h[b];
        uint32_t total;
        uint32_t before = block_exclusive_scan(s, wave_sum, total);
        for (uint32_t b = first; b < last; ++b) {
            const uint32_t v = h[b];
            h[b] = before;
            before += v;
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < kPer; ++r) {
            if (slot[r] == 0xffffffffu) continue;
            const uint32_t b = slot[r] / kBucketClusters;
            // (position in the chunk | slot << 13, record): the write loop then needs nothing but the row
            stage[h[b] + rank[r]] = make_uint2(uint32_t(r * kThreads + threadIdx.x) | (slot[r] << 13), first_rec[b] + rank[r]);
        }
        __syncthreads();
        // One 16-byte piece per thread and step (the d/4 pieces of the row, then the trailer), so that a wave
        // writes whole records side by side wherever a bucket's run is contiguous.
        constexpr int P = D / 4 + 1, U = 4;
        const uint32_t pieces = total * P;
        for (uint32_t g0 = 0; g0 < pieces; g0 += U * kThreads) {
            uint2 t[U];
            float4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) t[u] = stage[min(g0 + u * kThreads + threadIdx.x, pieces - 1) / P];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t q = min(g0 + u * kThreads + threadIdx.x, pieces - 1) % P;
                const uint32_t i = lo + (t[u].x & 8191u);
                if (q < D / 4) {
                    v[u] = reinterpret_cast<const float4*>(X + size_t(i) * D)[q];
                } else {
                    v[u] = make_float4(__uint_as_float(t[u].x >> 13), __uint_as_float(i), 0.0f, 0.0f);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t g = g0 + u * kThreads + threadIdx.x;
                if (g < pieces) reinterpret_cast<float4*>(records + size_t(t[u].y) * Record<D>::kBytes)[g % P] = v[u];
            }
        }
    }
}

// ---- 3'. the changed vectors only: two records each (third trailer word: 0 = add to the new cluster, 1 = take
// from the old one). Few records, so each lane writes its own straight to where its bucket's cursor points.
template <int D>
__global__ __launch_bounds__(kThreads) void bucket_scatter_delta_kernel(const float* __restrict__ X, uint32_t N,
                                                                        const uint32_t* __restrict__ idx,
                                                                        const uint32_t* __restrict__ prev,
                                                                        const uint32_t* __restrict__ changed, uint32_t K,
                                                                        const uint32_t* __restrict__ cinv,
                                                                        uint32_t nbuckets,
                                                                        const uint32_t* __restrict__ hist,
                                                                        const uint32_t* __restrict__ gtot,
                                                                        const uint32_t* __restrict__ base,
                                                                        char* __restrict__ records)
{
    __shared__ uint32_t cursor[kMaxBuckets];  // next free record of (bucket, this block)
    __shared__ uint16_t flagged[kDeltaChunk];
    __shared__ uint32_t wave_sum[kThreads / 64];
    const uint32_t blk = chunk_of_workgroup();
    for (uint32_t b = threadIdx.x; b < nbuckets; b += kThreads)
        cursor[b] = base[b] + gtot[size_t(blk / kBucketGroup) * nbuckets + b] + hist[size_t(blk) * nbuckets + b];
    __syncthreads();
    const uint32_t lo = blk * kDeltaChunk;
    for_each_flagged(changed, lo, N, flagged, wave_sum, [&](uint32_t i) {
        const uint32_t k_new = idx[i], k_old = prev[i];
        if (k_new == k_old || k_new >= K || k_old >= K) return;
        float4 row[D / 4];
#pragma unroll
        for (int q = 0; q < D / 4; ++q) row[q] = reinterpret_cast<const float4*>(X + size_t(i) * D)[q];
#pragma unroll
        for (uint32_t minus = 0; minus < 2; ++minus) {  // a record for the new cluster, one for the old
            const uint32_t slot = slot_of_code(minus ? k_old : k_new, cinv);
            const uint32_t pos = atomicAdd(&cursor[slot / kBucketClusters], 1u);
            char* rec = records + size_t(pos) * Record<D>::kBytes;
#pragma unroll
            for (int q = 0; q < D / 4; ++q) reinterpret_cast<float4*>(rec)[q] = row[q];
            *reinterpret_cast<uint4*>(rec + D * 4) = make_uint4(slot, i, minus, 0u);
        }
    });
}

// ---- 4. one workgroup per bucket: sums in LDS (component-major, so that the clusters of a bucket spread over
// all banks), then the means
template <int D>
__global__ __launch_bounds__(kThreads) void bucket_sum_kernel(const char* __restrict__ records,
                                                              const uint32_t* __restrict__ base, uint32_t N, uint32_t K,
                                                              const uint32_t* __restrict__ cperm, const float* prev,
                                                              float* out, uint32_t* counts_out, WsHeader* hdr, int mean,
                                                              long long* __restrict__ sums_ws,
                                                              uint32_t* __restrict__ counts_ws, int delta)
{
    __shared__ unsigned long long sum[D][kBucketClusters];
    __shared__ uint32_t cnt[kBucketClusters];
    for (uint32_t t = threadIdx.x; t < kBucketClusters * D; t += kThreads) (&sum[0][0])[t] = 0;
    if (threadIdx.x < kBucketClusters) cnt[threadIdx.x] = 0;
    __syncthreads();
    const int e = fixed_point_exp(hdr->absmax_bits, N);
    const uint32_t p0 = blockIdx.x * kBucketClusters;
    const uint32_t first = base[blockIdx.x], last = base[blockIdx.x + 1];
    for (uint32_t p = first + threadIdx.x; p < last; p += kThreads) {
        const char* rec = records + size_t(p) * Record<D>::kBytes;
        const uint2 tag = *reinterpret_cast<const uint2*>(rec + D * 4);
        const uint32_t local = (tag.x - p0) & (kBucketClusters - 1);
        const uint32_t minus = *reinterpret_cast<const uint32_t*>(rec + D * 4 + 8);  // 1: a vector that left the cluster
        float x[D];
        load_row<D>(reinterpret_cast<const float*>(rec), x);
#pragma unroll
        for (int j = 0; j < D; ++j) {
            const long long v = fixed_point_term(x[j], e);
            atomicAdd(&sum[j][local], static_cast<unsigned long long>(minus ? -v : v));  // two's complement: wraps like int64
        }
        atomicAdd(&cnt[local], minus ? 0xffffffffu : 1u);
    }
    __syncthreads();
    if (blockIdx.x == 0 && threadIdx.x == 0) hdr->fixed_point_exp = e;
    // cluster sizes first (one thread per cluster): the running totals stay in the workspace, where a later
    // iteration of the same fit adds its net change to them
    if (threadIdx.x < kBucketClusters && p0 + threadIdx.x < K) {
        const uint32_t k = cperm != nullptr ? cperm[p0 + threadIdx.x] : p0 + threadIdx.x;
        uint32_t n = cnt[threadIdx.x];
        if (delta) n += counts_ws[k];
        counts_ws[k] = n;
        cnt[threadIdx.x] = n;
        if (counts_out != nullptr) counts_out[k] = n;
    }
    __syncthreads();
    for (uint32_t t = threadIdx.x; t < kBucketClusters * D; t += kThreads) {
        const uint32_t local = t / D, j = t % D;
        if (p0 + local >= K) continue;
        const uint32_t k = cperm != nullptr ? cperm[p0 + local] : p0 + local;
        const size_t o = size_t(k) * D + j;
        long long isum = static_cast<long long>(sum[j][local]);
        if (delta) isum += sums_ws[o];
        sums_ws[o] = isum;
        const uint32_t n = cnt[local];
        const double total = ldexp(double(isum), -e);
        // mean: one fp64 division, one rounding to fp32; an empty cluster keeps its previous centroid
        out[o] = !mean ? float(total) : (n > 0 ? float(total / double(n)) : prev[o]);
    }
}

template <int D>
static void update_buckets_t(const float* X, uint32_t N, const uint32_t* idx, const uint32_t* prev_idx,
                             const uint32_t* changed, const float* prev, uint32_t K, float* out, uint32_t* counts_out,
                             const Workspace& w, bool norm_order, bool mean, hipStream_t s)
{
    const uint32_t nbuckets = (K + kBucketClusters - 1) / kBucketClusters;
    const bool delta = prev_idx != nullptr && changed != nullptr;
    const uint32_t chunk = delta ? kDeltaChunk : kBucketChunk;
    const uint32_t blocks = (N + chunk - 1) / chunk;
    const uint32_t* cinv = norm_order ? w.cinv : nullptr;
    const uint32_t* cperm = norm_order ? w.cperm : nullptr;
    hipLaunchKernelGGL(bucket_count_kernel, dim3(blocks), dim3(kThreads), 0, s, idx, delta ? prev_idx : nullptr, delta ? changed : nullptr, N, K,
                       cinv, nbuckets, w.bucket_hist, w.hdr);
    const uint32_t groups = (blocks + kBucketGroup - 1) / kBucketGroup;
    const uint32_t bwg = (nbuckets + kThreads - 1) / kThreads;
    hipLaunchKernelGGL(bucket_groupscan_kernel, dim3(bwg, groups), dim3(kThreads), 0, s, w.bucket_hist, blocks, nbuckets,
                       w.bucket_gtot);
    hipLaunchKernelGGL(bucket_base_kernel, dim3(1), dim3(kMaxBuckets), 0, s, w.bucket_gtot, groups, nbuckets, w.bucket_base);
    if (delta)
        hipLaunchKernelGGL(bucket_scatter_delta_kernel<D>, dim3(blocks), dim3(kThreads), 0, s, X, N, idx, prev_idx, changed, K,
                           cinv, nbuckets, w.bucket_hist, w.bucket_gtot, w.bucket_base, w.records);
    else
        hipLaunchKernelGGL(bucket_scatter_kernel<D>, dim3(blocks), dim3(kThreads), 0, s, X, N, idx, K, cinv, nbuckets,
                           w.bucket_hist, w.bucket_gtot, w.bucket_base, w.records);
    hipLaunchKernelGGL(bucket_sum_kernel<D>, dim3(nbuckets), dim3(kThreads), 0, s, w.records, w.bucket_base, N, K, cperm,
                       prev, out, counts_out, w.hdr, mean ? 1 : 0, w.sums, w.counts, delta ? 1 : 0);
}

hipError_t launch_update_buckets(const float* X, uint32_t N, uint32_t d, const uint32_t* idx, const float* prev,
                                 uint32_t K, float* out, uint32_t* counts_out, const Workspace& w, bool norm_order,
                                 bool mean, hipStream_t s, const uint32_t* prev_idx, const uint32_t* changed)
{
    if (K > kMaxBuckets * kBucketClusters || w.records == nullptr || (prev_idx != nullptr) != (changed != nullptr))
        return hipErrorInvalidValue;
    switch (d) {
        case 4: update_buckets_t<4>(X, N, idx, prev_idx, changed, prev, K, out, counts_out, w, norm_order, mean, s); break;
        case 8: update_buckets_t<8>(X, N, idx, prev_idx, changed, prev, K, out, counts_out, w, norm_order, mean, s); break;
        case 16: update_buckets_t<16>(X, N, idx, prev_idx, changed, prev, K, out, counts_out, w, norm_order, mean, s); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace cc
