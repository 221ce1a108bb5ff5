// M-step by cluster slices (Section 3.1: c_k <- mean of the vectors assigned to cluster k), for many vectors and
// K <= 65536: one pass over the codes, no copy of the vectors.
//
// The K x (d sums + count) accumulators do not fit one workgroup's LDS, but a slice of them does (4096 clusters at
// d = 4, 2048 at d = 8, 1024 at d = 16: 64-bit fixed-point sums, about 144 KB). So the clusters are cut into slices
// and the vectors into ranges, and workgroup (slice s, range r) - there are about as many as compute units - scans the
// codes of its range, fetches the rows whose code falls in its slice (1 in K / slice of them: a wave first packs the
// matching positions into a small LDS queue and then handles 64 of them at a time, so that no instruction runs with a
// handful of active lanes), and adds them into its LDS accumulators with integer atomics. The per-workgroup results go
// to the workspace and a second kernel adds the ranges of every cluster and divides.
//
// Every code is read once per slice, every row exactly once; nothing is written but the partial sums (37 MB at
// K = 65536, d = 4). Workgroups are numbered so that one XCD (they are dealt to the 8 XCDs in turn) owns whole ranges:
// its L2 then serves the repeated code reads and the cache lines whose rows belong to several slices. The sums are the same 64-bit integers as in the other formulations of
// the M-step, so the result is the same bits, whatever the scheduling.
//
// The same kernel serves the gradient of a layer's codebook (Sections 3.2-3.3: the sum of the weight gradient over the
// entries rebuilt from each codebook entry): there the rows are 16-bit numbers and the codes the layer's stored 16-bit
// codes, both read in place and converted as they are fetched (SRC below).
//
// Bound: one 16/32/64-byte row fetch per vector from a different cache line each - the L1 fill rate (about 0.4 lines
// per clock and compute unit), the same limit as the reconstruction's gathers - not HBM bandwidth.
#include <algorithm>
#include <type_traits>

#include "common.h"

namespace cc {

namespace {

constexpr int kThreads = 1024;            // 16 waves: what hides the latency of the row fetches
constexpr int kWaves = kThreads / 64;
constexpr uint32_t kQueue = 192;          // entries per wave: fewer than 64 left over + 128 new per round
constexpr uint32_t kTargetWorkgroups = 256;

// Where rows and codes come from: 0 = fp32 rows and 32-bit codes (the clustering), 1 = fp16 and 2 = bf16 rows with
// 16-bit codes (a layer's gradient): the numbering of cc_dtype.
template <int D, int SRC>
__device__ __forceinline__ void fetch_row(const void* __restrict__ X, size_t row, float (&v)[D])
{
    if constexpr (SRC == 0) {
        load_row<D>(static_cast<const float*>(X) + row * D, v);
    } else {
        uint32_t w[D / 2];  // two numbers per word, the lower-addressed one in the low half
        if constexpr (D == 4) {
            const uint2 t = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(X) + row * 4);
            w[0] = t.x; w[1] = t.y;
        } else {
#pragma unroll
            for (int q = 0; q < D / 8; ++q) {
                const uint4 t = reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(X) + row * D)[q];
                w[4 * q + 0] = t.x; w[4 * q + 1] = t.y; w[4 * q + 2] = t.z; w[4 * q + 3] = t.w;
            }
        }
#pragma unroll
        for (int p = 0; p < D / 2; ++p) {
            if constexpr (SRC == 2) {
                v[2 * p] = __uint_as_float(w[p] << 16);
                v[2 * p + 1] = __uint_as_float(w[p] & 0xffff0000u);
            } else {
                const uint16_t lo = uint16_t(w[p] & 0xffffu), hi = uint16_t(w[p] >> 16);
                v[2 * p] = float(__builtin_bit_cast(_Float16, lo));
                v[2 * p + 1] = float(__builtin_bit_cast(_Float16, hi));
            }
        }
    }
}

// Two consecutive codes, as one load: a uint2 of 32-bit codes, or one word of two 16-bit codes.
template <int SRC>
struct CodePair {
    using Word = typename std::conditional<SRC == 0, uint2, uint32_t>::type;
    using Code = typename std::conditional<SRC == 0, uint32_t, uint16_t>::type;
    static __device__ __forceinline__ Word load(const void* idx, size_t first) {
        return *reinterpret_cast<const Word*>(static_cast<const Code*>(idx) + first);
    }
    static __device__ __forceinline__ uint32_t one(const void* idx, size_t i) { return static_cast<const Code*>(idx)[i]; }
    static __device__ __forceinline__ uint32_t first(Word w) { if constexpr (SRC == 0) return w.x; else return w & 0xffffu; }
    static __device__ __forceinline__ uint32_t second(Word w) { if constexpr (SRC == 0) return w.y; else return w >> 16; }
};

template <int D>
struct Slice {
    static constexpr uint32_t kBits = D == 4 ? 12u : (D == 8 ? 11u : 10u);
    static constexpr uint32_t kClusters = 1u << kBits;
    static constexpr uint32_t kSumBytes = kClusters * D * 8;
    // a queue entry packs (position within the range, cluster within the slice) into 32 bits
    static constexpr uint32_t kMaxRange = 1u << (32 - kBits);
    static constexpr uint32_t kLdsBytes = kSumBytes + kClusters * 4;   // dynamic part; the queues are a static array
};

struct Cut {
    uint32_t slices, ranges;
};

template <int D>
Cut cut_of(uint32_t N, uint32_t K)
{
    Cut c;
    c.slices = (K + Slice<D>::kClusters - 1) / Slice<D>::kClusters;
    // about one workgroup per compute unit, and ranges short enough for the packed queue entries (128 of slack for
    // the rounding of the range length)
    const uint32_t by_entry = uint32_t((uint64_t(N) + Slice<D>::kMaxRange - 129) / (Slice<D>::kMaxRange - 128));
    c.ranges = std::max({1u, kTargetWorkgroups / c.slices, by_entry});
    return c;
}

// (slice, range) of a workgroup. Workgroups are dealt to the 8 XCDs in turn; XCD q takes the q-th contiguous share of
// the jobs in range-major order, i.e. all slices of a few ranges: the workgroups that scan the same codes and fetch
// rows from the same cache lines (a 128-byte line holds rows of several slices) then share one L2, so every line
// comes from memory once instead of once per slice.
__device__ __forceinline__ bool job_of_workgroup(uint32_t slices, uint32_t ranges, uint32_t& slice, uint32_t& range)
{
    const uint32_t jobs = slices * ranges, per_xcd = (jobs + 7) / 8;
    const uint32_t job = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
    slice = job % slices;
    range = job / slices;
    return job < jobs && blockIdx.x / 8 < per_xcd;
}

template <int D, int SRC>
__global__ __launch_bounds__(kThreads, 1) void sliced_accumulate_kernel(const void* __restrict__ X, uint32_t N,
                                                                     const void* __restrict__ idx, uint32_t K,
                                                                     uint32_t slices, uint32_t ranges, WsHeader* hdr,
                                                                     unsigned long long* __restrict__ part_sums,
                                                                     uint32_t* __restrict__ part_counts)
{
    using S = Slice<D>;
    using CP = CodePair<SRC>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned long long* sum = reinterpret_cast<unsigned long long*>(smem);              // [D][kClusters]
    uint32_t* cnt = reinterpret_cast<uint32_t*>(smem + S::kSumBytes);                   // [kClusters]
    // per-wave queues of matching positions. A static array, accessed through a plain pointer: a volatile or
    // re-cast pointer loses the LDS address space and turns every access into a flat one, which waits for all
    // outstanding global loads too. A wave's LDS instructions execute in order, so entries written by one lane are
    // seen by the lanes that read them in a later instruction.
    __shared__ uint32_t queues[kWaves * kQueue];
    uint32_t slice, range;
    if (!job_of_workgroup(slices, ranges, slice, range)) return;  // uniform over the workgroup
    for (uint32_t t = threadIdx.x; t < S::kClusters * D; t += kThreads) sum[t] = 0;
    for (uint32_t t = threadIdx.x; t < S::kClusters; t += kThreads) cnt[t] = 0;
    __syncthreads();

    const uint32_t k_lo = slice * S::kClusters;
    const uint32_t k_n = min(S::kClusters, K - k_lo);   // clusters of this slice
    // vectors of this range: a multiple of 128 each, so that every wave round starts on an 8-byte boundary of idx
    const uint32_t per = ((N + ranges - 1) / ranges + 127u) & ~127u;
    const uint32_t lo = min(uint64_t(range) * per, uint64_t(N)), hi = min(uint64_t(lo) + per, uint64_t(N));
    const int e = fixed_point_exp(hdr->absmax_bits, N);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t* q = queues + wave * kQueue;
    uint32_t len = 0, bad = 0;

    // The first n (<= 64) queued vectors are added to the accumulators in two steps, so that the latency of the row
    // fetches is spent scanning the next codes: fetch() reads the entries and requests the rows, commit() - called
    // when the next batch is ready, or at the end - converts and adds them.
    float px[D];
    uint32_t pclu = 0;
    bool pending = false, pactive = false;
    auto commit = [&]() {
        if (pending && pactive) {
#pragma unroll
            for (int j = 0; j < D; ++j) {
                const long long v = fixed_point_term(px[j], e);
                if (v != 0) atomicAdd(&sum[j * S::kClusters + pclu], static_cast<unsigned long long>(v));
            }
            atomicAdd(&cnt[pclu], 1u);
        }
        pending = false;
    };
    auto fetch = [&](uint32_t n) {
        commit();
        pactive = uint32_t(lane) < n;
        if (pactive) {
            const uint32_t ent = q[lane];  // (position within the range, cluster within the slice)
            pclu = ent & (S::kClusters - 1);
            fetch_row<D, SRC>(X, size_t(lo + (ent >> S::kBits)), px);
        }
        pending = true;
    };
    // moves what is left after a batch of 64 to the front of the queue (fewer than 128 entries)
    auto shift = [&]() {
        uint32_t t0 = 0, t1 = 0;
        const bool m0 = 64u + lane < len, m1 = 128u + lane < len;
        if (m0) t0 = q[64 + lane];
        if (m1) t1 = q[128 + lane];
        __builtin_amdgcn_wave_barrier();
        if (m0) q[lane] = t0;
        if (m1) q[64 + lane] = t1;
        __builtin_amdgcn_wave_barrier();
        len -= 64;
    };
    // one code per lane: queue it if it belongs to this slice. `rel` = position within the range.
    auto scan = [&](uint32_t c, uint32_t rel) {
        const uint32_t local = c - k_lo;
        const bool match = local < k_n;   // a code below k_lo wraps to a huge value
        const unsigned long long m = __ballot(match);
        if (match) {
            const uint32_t pos = __builtin_amdgcn_mbcnt_hi(uint32_t(m >> 32), __builtin_amdgcn_mbcnt_lo(uint32_t(m), len));
            q[pos] = (rel << S::kBits) | local;
        }
        len += uint32_t(__popcll(m));
    };
    const bool count_bad = slice == 0;  // codes >= K belong to no slice: the workgroups of slice 0 count them

    // U rounds of 128 codes per wave are requested before the first is looked at: the LDS accumulators allow one
    // workgroup per compute unit, so nothing else hides the latency of the code reads. Whole blocks of U rounds
    // take the loop without range checks; the last, partial block of a wave checks every position.
    constexpr uint32_t U = 8, kRound = kWaves * 128u;
    uint32_t base = lo + wave * 128u;
    auto whole_block = [&](uint32_t b) { return b + (U - 1) * kRound + 128u <= hi; };
    typename CP::Word code[U], ahead[U];
    if (whole_block(base)) {
#pragma unroll
        for (uint32_t r = 0; r < U; ++r) ahead[r] = CP::load(idx, size_t(base) + r * kRound + 2u * lane);
    }
    for (; whole_block(base); base += kRound * U) {
#pragma unroll
        for (uint32_t r = 0; r < U; ++r) code[r] = ahead[r];
        if (whole_block(base + kRound * U)) {  // the block after this one is requested before this one is looked at
#pragma unroll
            for (uint32_t r = 0; r < U; ++r)
                ahead[r] = CP::load(idx, size_t(base) + kRound * U + r * kRound + 2u * lane);
        }
#pragma unroll
        for (uint32_t r = 0; r < U; ++r) {
            const uint32_t rel = base - lo + r * kRound + 2u * lane;
            const uint32_t c0 = CP::first(code[r]), c1 = CP::second(code[r]);
            scan(c0, rel);
            scan(c1, rel + 1);
            if (count_bad) bad += (c0 >= K ? 1u : 0u) + (c1 >= K ? 1u : 0u);
            __builtin_amdgcn_wave_barrier();
            while (len >= 64) {
                fetch(64);
                shift();
            }
        }
    }
    for (; base < hi; base += kRound) {
#pragma unroll
        for (uint32_t u = 0; u < 2; ++u) {
            const uint32_t i = base + 2u * lane + u;
            const bool live = i < hi;
            const uint32_t c = live ? CP::one(idx, i) : k_lo + k_n;   // a code of the next slice: matches nothing here
            scan(c, i - lo);
            if (count_bad) bad += (live && c >= K) ? 1u : 0u;
        }
        __builtin_amdgcn_wave_barrier();
        while (len >= 64) {
            fetch(64);
            shift();
        }
    }
    fetch(len);
    commit();
    if (bad) atomicAdd(&hdr->skipped_vectors, static_cast<unsigned long long>(bad));
    __syncthreads();
    const size_t job = size_t(slice) * ranges + range;
    unsigned long long* ps = part_sums + job * (S::kClusters * D);
    uint32_t* pc = part_counts + job * S::kClusters;
    for (uint32_t t = threadIdx.x; t < S::kClusters * D; t += kThreads) ps[t] = sum[t];
    for (uint32_t t = threadIdx.x; t < S::kClusters; t += kThreads) pc[t] = cnt[t];
}

// Adds the ranges of every cluster (integers: any order gives the same bits; this one is fixed anyway), leaves the
// totals in the workspace and writes the means (or, mean = 0, the plain sums). An empty cluster keeps prev.
template <int D>
__global__ __launch_bounds__(256) void sliced_finalize_kernel(const unsigned long long* __restrict__ part_sums,
                                                              const uint32_t* __restrict__ part_counts, uint32_t ranges,
                                                              const float* prev, float* out, uint32_t* counts_out, uint32_t K,
                                                              uint32_t N, WsHeader* hdr, int mean, long long* __restrict__ sums_ws,
                                                              uint32_t* __restrict__ counts_ws)
{
    using S = Slice<D>;
    const uint32_t t = blockIdx.x * 256 + threadIdx.x;   // (component, cluster): clusters vary fastest
    const int e = fixed_point_exp(hdr->absmax_bits, N);
    if (t == 0) hdr->fixed_point_exp = e;
    if (t >= K * D) return;
    const uint32_t j = t / K, k = t % K;
    const uint32_t slice = k / S::kClusters, local = k % S::kClusters;
    long long isum = 0;
    uint32_t n = 0;
    for (uint32_t r = 0; r < ranges; ++r) {
        const size_t job = size_t(slice) * ranges + r;
        isum += static_cast<long long>(part_sums[job * (S::kClusters * D) + j * S::kClusters + local]);
        n += part_counts[job * S::kClusters + local];
    }
    const size_t o = size_t(k) * D + j;
    sums_ws[o] = isum;
    if (j == 0) {
        counts_ws[k] = n;
        if (counts_out != nullptr) counts_out[k] = n;
    }
    const double total = ldexp(double(isum), -e);
    out[o] = !mean ? float(total) : (n > 0 ? float(total / double(n)) : prev[o]);
}

template <int D, int SRC>
hipError_t update_sliced_t(const void* X, uint32_t N, const void* idx, const float* prev, uint32_t K, float* out,
                           uint32_t* counts_out, const Workspace& w, bool mean, hipStream_t s)
{
    using S = Slice<D>;
    const Cut c = cut_of<D>(N, K);
    const size_t jobs = size_t(c.slices) * c.ranges;
    unsigned long long* part_sums = reinterpret_cast<unsigned long long*>(w.records);
    uint32_t* part_counts = reinterpret_cast<uint32_t*>(w.records + jobs * S::kSumBytes);
    static bool lds_set = false;
    if (!lds_set) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&sliced_accumulate_kernel<D, SRC>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, int(S::kLdsBytes));
        if (e != hipSuccess) return e;
        lds_set = true;
    }
    hipLaunchKernelGGL((sliced_accumulate_kernel<D, SRC>), dim3(uint32_t(8 * ((jobs + 7) / 8))), dim3(kThreads), S::kLdsBytes, s, X, N, idx, K,
                       c.slices, c.ranges, w.hdr, part_sums, part_counts);
    hipLaunchKernelGGL(sliced_finalize_kernel<D>, dim3((K * D + 255) / 256), dim3(256), 0, s, part_sums, part_counts, c.ranges,
                       prev, out, counts_out, K, N, w.hdr, mean ? 1 : 0, w.sums, w.counts);
    return hipGetLastError();
}

template <int D>
size_t sliced_bytes_t(uint32_t N, uint32_t K)
{
    const Cut c = cut_of<D>(N, K);
    return size_t(c.slices) * c.ranges * (Slice<D>::kSumBytes + Slice<D>::kClusters * 4);
}

}  // namespace

// Whether the M-step by slices applies: enough vectors that one pass per slice over the codes pays, and a workspace
// whose record buffer (2 N records) holds the per-workgroup partial sums.
bool update_sliced_applies(uint32_t N, uint32_t d, uint32_t K, const Workspace& w)
{
    if (!w.bucket_ok || w.records == nullptr || N < (1u << 20)) return false;
    const size_t have = size_t(N) * 2 * (4 * d + 16);
    const size_t need = d == 4 ? sliced_bytes_t<4>(N, K) : (d == 8 ? sliced_bytes_t<8>(N, K) : sliced_bytes_t<16>(N, K));
    return need <= have;
}

// in `out` may alias `prev`; `out` must not alias X. Sums and counts are left in w.sums / w.counts.
hipError_t launch_update_sliced(const float* X, uint32_t N, uint32_t d, const uint32_t* idx, const float* prev, uint32_t K,
                                float* out, uint32_t* counts_out, const Workspace& w, bool mean, hipStream_t s)
{
    if (!update_sliced_applies(N, d, K, w)) return hipErrorInvalidValue;
    switch (d) {
        case 4: return update_sliced_t<4, 0>(X, N, idx, prev, K, out, counts_out, w, mean, s);
        case 8: return update_sliced_t<8, 0>(X, N, idx, prev, K, out, counts_out, w, mean, s);
        case 16: return update_sliced_t<16, 0>(X, N, idx, prev, K, out, counts_out, w, mean, s);
        default: return hipErrorInvalidValue;
    }
}

// The sums (not the means) of 16-bit rows by 16-bit code, read in place: rows [N * d] fp16 (dtype 1) or bf16 (2),
// 16-byte aligned; codes [N], 4-byte aligned. The input scan of the rows (launch_scan_inputs16) must have run on this
// workspace since the last header reset. Same fixed-point sums as launch_update on the converted rows: same bits.
hipError_t launch_sum_rows16_sliced(const void* rows, int dtype, uint32_t N, uint32_t d, const uint16_t* codes, uint32_t K,
                                    float* out, const Workspace& w, hipStream_t s)
{
    if (!update_sliced_applies(N, d, K, w) || (dtype != 1 && dtype != 2)) return hipErrorInvalidValue;
    const bool bf = dtype == 2;
    switch (d) {
        case 4: return bf ? update_sliced_t<4, 2>(rows, N, codes, nullptr, K, out, nullptr, w, false, s)
                          : update_sliced_t<4, 1>(rows, N, codes, nullptr, K, out, nullptr, w, false, s);
        case 8: return bf ? update_sliced_t<8, 2>(rows, N, codes, nullptr, K, out, nullptr, w, false, s)
                          : update_sliced_t<8, 1>(rows, N, codes, nullptr, K, out, nullptr, w, false, s);
        case 16: return bf ? update_sliced_t<16, 2>(rows, N, codes, nullptr, K, out, nullptr, w, false, s)
                           : update_sliced_t<16, 1>(rows, N, codes, nullptr, K, out, nullptr, w, false, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace cc
