// Internal declarations shared by the translation units of libcluscomp (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <algorithm>

namespace cc {

// bytes of the radix sort's histogram buffer for n elements (sort.hip)
size_t sort_hist_bytes(uint64_t n);

constexpr uint32_t kMaxK = 1u << 24;

// Device time of the library's own kernels, for callers that ask for it (cc_profile in the public header): a pool
// of HIP events created once; a scope records one event before and one after the launches it brackets, on the
// stream of the call. Slots follow cc_profile_slot. A NULL profile, a slot outside the caller's mask or a full pool
// turns a scope into a no-op.
struct Profile;
struct ProfileScope {
    ProfileScope(Profile* p, int slot, hipStream_t s);
    ~ProfileScope();
    ProfileScope(const ProfileScope&) = delete;
    ProfileScope& operator=(const ProfileScope&) = delete;
    Profile* p_;
    hipStream_t s_;
    int record_;
};
enum ProfileSlot : int { kProfEstepF16 = 0, kProfEstepF32 = 1, kProfEstepDirect = 2, kProfRefine = 3, kProfMstep = 4,
                         kProfOrder = 5, kProfSlots = 6 };

// Device-side bookkeeping at the start of the workspace (one 256-byte slot).
struct WsHeader {
    uint32_t absmax_bits;      // max over all inputs of the fp32 bit pattern of |x|
    uint32_t refine_count;     // length of the refine list written by the last matrix-core assign
    uint32_t x_not_f16;        // != 0: some |x| >= 2^15, or some |x| >= 2^-14 is not an fp16 number
    uint32_t cmax_bits;        // max over the current codebook of the fp32 bit pattern of |c|
    unsigned long long refined_vectors;
    unsigned long long skipped_vectors;
    unsigned long long assign_calls;
    unsigned long long window_stages;   // sum over 512-vector tiles of the codebook stages they had to score
    unsigned long long window_total;    // what that sum would be without pruning
    int32_t fixed_point_exp;
    uint32_t x_nonfinite;      // != 0: some input is Inf or NaN (the sums then skip such components)
};

// Survives between calls on the same workspace (not touched by the per-call header reset): whether the
// norm-ordered codes of the previous E-step may serve as a hint. A hint never affects results, only
// how much of the codebook has to be scored.
struct WsPersist {
    unsigned long long magic;
    uint32_t N, d, K;
    uint32_t hint_valid;
};

// Carved view of the caller's workspace.
struct Workspace {
    uint32_t d;                // sub-vector length the kernels run at: the caller's, rounded up to 4, 8 or 16
    bool padded;               // the caller's length differs: the kernels see zero-padded copies
    float* xpad;               // [N*d]  padded vectors   (only if padded)
    float* cpad;               // [K*d]  padded centroids (only if padded)
    WsHeader* hdr;
    float* cnorm;              // [K]    ||c_k||^2
    long long* sums;           // [K*d]  fixed-point cluster sums
    uint32_t* counts;          // [K]
    double* partials;          // [partial_slots] per-block partial objective
    float* dmin;               // [N]    ||x_i - c_idx_i||^2 of the last assign (fp32, direct form)
    float* packed;             // codebook re-laid out as matrix-core operand tiles (+ ||c||^2)
    uint32_t* refine_list;     // [refine_cap] ids of vectors to re-decide in direct form
    // norm ordering for the pruned E-step
    WsPersist* persist;
    float* xsorted;            // [N*d]  the vectors in ascending-norm order
    uint32_t* idx_sorted;      // [N]    codes in that order (also the next call's hint)
    uint32_t* idx_prev;        // [N]    the previous iteration's code of every vector flagged in `changed` (incremental M-step)
    uint32_t* changed;         // [ceil(N/32)] one bit per ordered vector: its code may differ from the previous iteration's
    uint32_t* vperm;           // [N]    input position of the p-th vector in norm order
    uint32_t* vperm_tmp;       // [N]
    uint16_t* vkeys;           // [N]    norm keys (sorted after the sort)
    uint16_t* vkeys_tmp;       // [N]
    float* csorted;            // [K*d]  the centroids in ascending-norm order
    uint32_t* cperm;           // [K]    centroid index of the p-th centroid in norm order
    uint32_t* cperm_tmp;       // [K]
    uint32_t* cinv;            // [K]    position of centroid k in norm order (inverse of cperm)
    uint16_t* ckeys;           // [K]
    uint16_t* ckeys_tmp;       // [K]
    uint32_t* key_starts;      // [65537] first norm-ordered centroid position with ordering key >= v
    uint32_t* sort_hist;       // [256 * sort blocks]
    uint2* windows;            // [ceil(N/512)][kWinStride] window list (runs of codebook stages) per 512-vector tile
    // M-step by buckets (K <= kMaxBuckets * kBucketClusters)
    char* records;             // [2N] x (4d + 16) bytes: the vectors, each with its code, grouped by bucket
    uint32_t* bucket_hist;     // [blocks][buckets] members of each bucket in each block of kBucketChunk vectors
    uint32_t* bucket_gtot;     // [groups of kBucketGroup blocks][buckets]
    uint32_t* bucket_base;     // [buckets + 1] first record of each bucket
    bool bucket_ok;
    uint32_t refine_cap;
    uint32_t partial_slots;
    uint32_t packed_tiles;     // number of 32-centroid tiles in `packed` (K rounded up, padded)
    size_t bytes;
};

constexpr uint32_t kTileCentroids = 32;   // centroids per matrix-core tile
constexpr uint32_t kGroupTiles = 2;       // tiles per tracking group of the matrix-core E-step
constexpr uint32_t kStageTilesMax = 8;    // the packed codebook is padded to whole LDS stages of this many tiles
constexpr uint32_t kStageTiles = 4;       // tiles per LDS stage of the matrix-core E-step kernels
constexpr uint32_t kWinQuad = kTileCentroids;  // window lists count runs in tiles = 32 positions; runs never share a stage
constexpr int kWinSlots = 32;             // most runs a window list can hold (one per norm shell)
// Vectors (neighbours in the norm order) that share one window list: what one workgroup of the windowed kernels
// scores (4 waves x 4 tiles of 32). Half of that gives tighter hulls but halves the work per staged codebook tile:
// measured 29.0 -> 31.9 ms per cfg3 fit.
constexpr uint32_t kWinTile = 512;
constexpr int kWinStride = kWinSlots + 1; // uint2 entries per 512-vector tile: (count, -), then the runs
constexpr uint32_t kBucketClusters = 64;  // M-step by buckets: consecutive clusters summed by one workgroup
constexpr uint32_t kMaxBuckets = 1024;    // so K <= 65536 for that path
constexpr uint32_t kBucketGroup = 64;     // blocks per group in the two-level scan of the bucket histogram
constexpr uint32_t kBucketChunk = 4096;   // vectors per workgroup in its counting and scatter passes
constexpr uint32_t kDeltaChunk = 16384;   // the same for an incremental pass, which looks only at the flagged vectors

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

// Lays the arrays out behind `base` (which may be NULL for a pure size query).
inline Workspace carve(void* base, uint64_t N, uint32_t d_caller, uint32_t K)
{
    Workspace w{};
    const uint32_t d = d_caller <= 4 ? 4u : (d_caller <= 8 ? 8u : 16u);
    w.d = d;
    w.padded = d != d_caller;
    char* p = static_cast<char*>(base);
    size_t off = 0;
    auto take = [&](size_t bytes) { char* q = p ? p + off : nullptr; off += align256(bytes); return q; };
    static_assert(sizeof(WsHeader) <= 128 && sizeof(WsPersist) <= 128, "header slot layout");
    char* slot = take(256);
    w.hdr = reinterpret_cast<WsHeader*>(slot);
    w.persist = reinterpret_cast<WsPersist*>(slot ? slot + 128 : nullptr);
    w.cnorm = reinterpret_cast<float*>(take(size_t(K) * 4));
    w.sums = reinterpret_cast<long long*>(take(size_t(K) * d * 8));
    w.counts = reinterpret_cast<uint32_t*>(take(size_t(K) * 4));
    w.partial_slots = 1024;
    w.partials = reinterpret_cast<double*>(take(size_t(w.partial_slots) * 8));
    w.dmin = reinterpret_cast<float*>(take(size_t(N) * 4));
    const uint32_t stage = kTileCentroids * kStageTilesMax;
    w.packed_tiles = uint32_t((uint64_t(K) + stage - 1) / stage) * kStageTilesMax;
    // per centroid: fp32 operands + norm take 4(d+1) bytes; the fp16-split operands take up to 6d+4 bytes
    w.packed = reinterpret_cast<float*>(take(size_t(w.packed_tiles) * kTileCentroids * (6 * d + 16)));
    w.refine_cap = uint32_t(N / 8 + 4096);
    w.refine_list = reinterpret_cast<uint32_t*>(take(size_t(w.refine_cap) * 4));
    w.xsorted = reinterpret_cast<float*>(take(size_t(N) * d * 4));
    w.idx_sorted = reinterpret_cast<uint32_t*>(take(size_t(N) * 4));
    w.idx_prev = reinterpret_cast<uint32_t*>(take(size_t(N) * 4));
    w.changed = reinterpret_cast<uint32_t*>(take((size_t(N) / 32 + 1) * 4));
    w.vperm = reinterpret_cast<uint32_t*>(take(size_t(N) * 4));
    w.vperm_tmp = reinterpret_cast<uint32_t*>(take(size_t(N) * 4));
    w.vkeys = reinterpret_cast<uint16_t*>(take(size_t(N) * 2));
    w.vkeys_tmp = reinterpret_cast<uint16_t*>(take(size_t(N) * 2));
    w.csorted = reinterpret_cast<float*>(take(size_t(K) * d * 4));
    w.cperm = reinterpret_cast<uint32_t*>(take(size_t(K) * 4));
    w.cperm_tmp = reinterpret_cast<uint32_t*>(take(size_t(K) * 4));
    w.cinv = reinterpret_cast<uint32_t*>(take(size_t(K) * 4));
    w.ckeys = reinterpret_cast<uint16_t*>(take(size_t(K) * 2));
    w.ckeys_tmp = reinterpret_cast<uint16_t*>(take(size_t(K) * 2));
    w.key_starts = reinterpret_cast<uint32_t*>(take(size_t(65537) * 4));
    // histogram rows + 256 totals, for the vectors' sort and for the centroids' (whose blocks are smaller)
    w.sort_hist = reinterpret_cast<uint32_t*>(take(std::max(sort_hist_bytes(N), sort_hist_bytes(K))));
    w.windows = reinterpret_cast<uint2*>(take((size_t(N) / kWinTile + 1) * kWinStride * 8));
    if (w.padded) {
        w.xpad = reinterpret_cast<float*>(take(size_t(N) * d * 4));
        w.cpad = reinterpret_cast<float*>(take(size_t(K) * d * 4));
    }
    w.bucket_ok = K <= kMaxBuckets * kBucketClusters && N < (uint64_t(1) << 31);  // record positions are 32-bit
    if (w.bucket_ok) {
        const size_t buckets = (size_t(K) + kBucketClusters - 1) / kBucketClusters;
        // 2N records: an incremental M-step writes two records (plus, minus) per vector whose code changed, and
        // nothing bounds how many change in one iteration
        w.records = take(size_t(N) * 2 * (4 * d + 16));
        w.bucket_hist = reinterpret_cast<uint32_t*>(take(buckets * (size_t(N) / kBucketChunk + 1) * 4));
        w.bucket_gtot = reinterpret_cast<uint32_t*>(take(buckets * (size_t(N) / kBucketChunk / kBucketGroup + 1) * 4));
        w.bucket_base = reinterpret_cast<uint32_t*>(take((buckets + 1) * 4));
    }
    w.bytes = off;
    return w;
}

// ---- launchers (each enqueues on `s` and returns the launch status) -------------------------------

// Direct-form E-step over all N vectors; dmin may be NULL. With gate != NULL the kernel does nothing
// unless *gate > gate_limit (used as the overflow path of the matrix-core E-step).
hipError_t launch_assign_direct(const float* X, uint32_t N, uint32_t d, const float* C, uint32_t K,
                                uint32_t* idx, float* dmin, const uint32_t* gate, uint32_t gate_limit,
                                hipStream_t s, Profile* profile = nullptr);

// Which inputs a gated kernel runs for (decided on the device from WsHeader::x_not_f16).
// kGateNoHint (a flag on top of the three) additionally requires that the workspace holds no usable hint.
enum Gate : int { kGateIfF16 = 0, kGateIfNotF16 = 1, kGateAlways = 2, kGateNoHint = 4 };
__device__ __forceinline__ bool gate_open(const WsHeader* hdr, int gate)
{
    if (gate & kGateNoHint) {
        // the persistent state sits in the second half of the header's 256-byte slot
        const WsPersist* persist = reinterpret_cast<const WsPersist*>(reinterpret_cast<const char*>(hdr) + 128);
        if (persist->hint_valid != 0) return false;
    }
    const int base = gate & 3;
    return base == kGateAlways || (base == kGateIfF16) == (hdr->x_not_f16 == 0);
}

// One scoring pass of a matrix-core E-step kernel.
struct EStep {
    const float* X;             // vectors to score (input order, or the norm-ordered copy)
    uint32_t N;
    const float* pack_rows;     // centroid rows the packed codebook is built from ...
    const uint32_t* pack_perm;  // ... through this position -> row map (NULL = identity)
    const float* rows;          // centroid rows in packed order, for the direct-form index recovery ...
    const uint32_t* row_ids;    // ... and the centroid index of each packed position (NULL = identity)
    uint32_t K;                 // rows in this codebook
    void* packed;               // operand tiles
    uint32_t packed_tiles;
    const uint2* windows;       // per 512-vector tile window list (NULL = whole codebook)
    uint32_t* idx;              // codes out
    bool accumulate;            // also add every vector to the cluster sums/counts of its provisional code
    bool hint_only;             // only write codes: no guard band, no distances, no refine list
    uint32_t* prev_out;         // with `changed`: where the code that idx held before goes, for every vector flagged there
    uint32_t* changed;          // NULL, or one bit per vector, set where the code differs from what idx held or is not final yet
    int gate;
    Profile* profile;           // NULL, or where the scoring kernel's device time is recorded
};

// Matrix-core E-step, fp32 MFMA: packs the codebook and runs the scoring kernel (provisional idx,
// w.dmin and the refine list). Must be followed by launch_refine.
hipError_t launch_assign_mfma_f32(const EStep& e, uint32_t d, const Workspace& w, hipStream_t s);

// Matrix-core E-step for fp16-representable inputs: centroids split into three fp16 parts so that
// every product is exact, scored with the fp16 MFMA. Same outputs as the fp32 variant.
hipError_t launch_assign_mfma_f16(const EStep& e, uint32_t d, const Workspace& w, hipStream_t s);

// Norm ordering (pruned E-step): vectors once per call, centroids + per-tile windows once per E-step,
// and the codes back to input order afterwards.
// drop_hint = true forgets the codes a previous call left in the workspace (a fit starts cold).
hipError_t launch_sort_vectors(const float* X, uint32_t N, uint32_t d, uint32_t K, const Workspace& w, bool drop_hint,
                               hipStream_t s);
hipError_t launch_sort_centroids(const float* C, uint32_t d, uint32_t K, const Workspace& w, hipStream_t s);
hipError_t launch_windows(const float* C, uint32_t N, uint32_t d, uint32_t K, const Workspace& w, float guess,
                          hipStream_t s);
hipError_t launch_unpermute(uint32_t N, uint32_t* idx, const Workspace& w, hipStream_t s);

// Re-decides the listed guard-band vectors over all K centroids in direct form; if the list
// overflowed, re-decides everything in direct form. With fix_sums = true the cluster sums/counts that
// the scoring kernel accumulated are corrected for every vector whose code changed (or rebuilt from
// scratch on overflow).
// With norm_ordered = true (X = w.xsorted, idx = w.idx_sorted) only each vector's window is searched and
// the codes are flagged as a usable hint for the next call.
hipError_t launch_refine(const float* X, uint32_t N, uint32_t d, const float* C, uint32_t K, uint32_t* idx,
                         const Workspace& w, bool fix_sums, bool norm_ordered, hipStream_t s);

// Scans the inputs: max |x| and whether every x is exactly representable in fp16.
hipError_t launch_scan_inputs(const float* X, uint64_t n_floats, WsHeader* hdr, hipStream_t s);

// *out = sum_i dmin[i] in fp64 with a fixed reduction shape.
hipError_t launch_reduce_dmin(const float* dmin, uint32_t N, double* partials, uint32_t partial_slots,
                              double* out, hipStream_t s);

// Header bookkeeping.
hipError_t launch_reset_header(WsHeader* hdr, hipStream_t s);
hipError_t launch_bump_assign_calls(WsHeader* hdr, hipStream_t s);

// M-step = zero the accumulators, accumulate, finalize. With gate != NULL a gated launch does nothing
// unless *gate > gate_limit (the refine-overflow path).
hipError_t launch_zero_accumulators(const Workspace& w, uint32_t K, uint32_t d, const uint32_t* gate,
                                    uint32_t gate_limit, hipStream_t s);
hipError_t launch_accumulate(const float* X, uint32_t N, uint32_t d, const uint32_t* idx, uint32_t K,
                             const Workspace& w, const uint32_t* gate, uint32_t gate_limit, hipStream_t s);
// M-step by buckets (K <= 65536): counts, scatter into per-bucket records, LDS sums, means (and counts_out if
// not NULL) in one go. Codes >= K are skipped and counted in WsHeader::skipped_vectors. norm_order = true
// buckets the clusters by their position in the norm order left by launch_sort_centroids (w.cinv, w.cperm).
// mean = false writes the plain sums (0 for an empty cluster) instead of the means. The integer sums and the
// counts are left in w.sums / w.counts. prev_idx != NULL: those already hold the sums and counts of the codes
// prev_idx; only the vectors whose code differs are moved (bit-identical to a recomputation from idx). That needs
// `changed` too, one bit per vector: prev_idx is only read, and only needs to be valid, where the bit is set, and a
// vector whose bit is clear must have kept its code.
hipError_t launch_update_buckets(const float* X, uint32_t N, uint32_t d, const uint32_t* idx, const float* prev,
                                 uint32_t K, float* out, uint32_t* counts_out, const Workspace& w, bool norm_order,
                                 bool mean, hipStream_t s, const uint32_t* prev_idx = nullptr,
                                 const uint32_t* changed = nullptr);
// M-step by cluster slices (update_sliced.hip): one pass over the codes per slice of the clusters, LDS accumulators,
// no copy of the vectors; for N >= 2^20 and K <= 65536. Same integer sums (left in w.sums / w.counts) and the same
// result bits as the other formulations. `out` may alias `prev`.
bool update_sliced_applies(uint32_t N, uint32_t d, uint32_t K, const Workspace& w);
// Sums (not means) of 16-bit rows (dtype 1 = fp16, 2 = bf16; 16-byte aligned) by 16-bit code (4-byte aligned), both read
// in place; needs update_sliced_applies(N, d, K, w) and launch_scan_inputs16 on the same workspace first.
hipError_t launch_sum_rows16_sliced(const void* rows, int dtype, uint32_t N, uint32_t d, const uint16_t* codes, uint32_t K,
                                    float* out, const Workspace& w, hipStream_t s);
hipError_t launch_scan_inputs16(const void* X, int dtype, uint64_t n, WsHeader* hdr, hipStream_t s);
hipError_t launch_update_sliced(const float* X, uint32_t N, uint32_t d, const uint32_t* idx, const float* prev, uint32_t K,
                                float* out, uint32_t* counts_out, const Workspace& w, bool mean, hipStream_t s);
// out[i][j] = j < d_in ? in[i][j] : 0 for rows of d_out >= d_in floats, and the reverse (drop the tail).
hipError_t launch_pad_rows(const float* in, uint32_t n, uint32_t d_in, uint32_t d_out, float* out, hipStream_t s);
hipError_t launch_unpad_rows(const float* in, uint32_t n, uint32_t d_in, uint32_t d_out, float* out, hipStream_t s);
hipError_t launch_finalize(const float* prev, float* out, uint32_t* counts_out, uint32_t K, uint32_t d, uint32_t N,
                           const Workspace& w, bool mean, hipStream_t s);
hipError_t launch_update(const float* X, uint32_t N, uint32_t d, const uint32_t* idx, const float* prev,
                         uint32_t K, float* out, uint32_t* counts_out, const Workspace& w, bool mean, hipStream_t s);

// ---- the compressed linear layer (layer.hip); dtype: 0 = fp32, 1 = fp16, 2 = bf16
hipError_t launch_layer_vectors(const void* weight, int dtype, uint32_t out_features, uint32_t in_features, uint32_t g,
                                float* vectors, hipStream_t s);
hipError_t launch_layer_pack_codebook(const float* centroids, size_t n, void* codebook, int dtype, hipStream_t s);
hipError_t launch_layer_pack_codes(const uint32_t* idx, uint64_t n, uint32_t K, uint16_t* codes, hipStream_t s);
hipError_t launch_layer_weight(const void* codebook, int dtype, uint32_t K, uint32_t g, const uint16_t* codes,
                               uint32_t in_features, uint32_t out_features, void* weight, hipStream_t s);
// y = x . W(codebook, codes) (+ bias); `partial` holds layer_forward_splits(...) * M * out_features floats if that
// count is above 1
uint32_t layer_forward_splits(uint64_t M, uint32_t in_features, uint32_t out_features);
bool layer_forward_few_rows(uint64_t M, uint32_t g);   // decode-time route of launch_layer_forward
uint32_t layer_forward_few_rows_max_splits();
hipError_t launch_layer_forward(const void* x, uint32_t M, const void* codebook, int dtype, uint32_t K, uint32_t g,
                                const uint16_t* codes, uint32_t in_features, uint32_t out_features, const void* bias,
                                void* y, float* partial, hipStream_t s);
// ---- codebook gradient from a prepared order of the codes (layer_grad_plan.hip); sort helpers from sort.hip
hipError_t launch_sort_u16(uint16_t* keys_a, uint32_t* ids_a, uint16_t* keys_b, uint32_t* ids_b, uint32_t n, uint32_t* hist,
                           hipStream_t s);
size_t layer_grad_plan_bytes(uint64_t num_codes, uint32_t K);
size_t layer_grad_plan_build_bytes(uint64_t num_codes);
size_t layer_grad_planned_bytes(uint64_t num_codes, uint32_t K, uint32_t g);
hipError_t launch_layer_grad_plan(const uint16_t* codes, uint32_t n, uint32_t K, void* plan, void* workspace, hipStream_t s);
hipError_t launch_layer_grad_planned(const void* grad, int dtype, uint32_t in_features, uint32_t out_features, uint32_t K,
                                     uint32_t g, uint32_t n, const void* plan, float* grad_codebook, void* workspace,
                                     hipStream_t s);
// ---- prefill-sized batches (layer_gemm.hip): W rebuilt into memory, then one dense product on the matrix cores
// From where on the rebuilt-weight route is the faster one. The fused kernels repeat their gathers per row tile (32,
// 64, 96, ... rows), the rebuild costs the same for any number of rows (58 us for 45 M weights). Measured on
// 4096 x 4096, 4096 x 11008, 11008 x 4096 and 8192 x 8192 (bf16, K = 65536, g = 4; fused / rebuilt + product, us):
// 16-bit codebook: 4096 x 4096 at 64 rows 40 / 51, at 96 rows 59 / 53; 4096 x 11008 at 32 rows 71 / 94, at 48 rows
// 108 / 94; 11008 x 4096 at 64 rows 73 / 94, at 96 rows 121 / 97; 8192 x 8192 at 64 rows 99 / 130, at 96 rows 165 / 133.
// 4-bit codebook (the integer codebook is expanded first, + 5 us): 4096 x 4096 at 32 rows 49 / 55, at 48 rows 58 / 55;
// 4096 x 11008 at 8 rows 56 / 96, at 16 rows 109 / 97; 11008 x 4096 at 16 rows 85 / 96, at 24 rows 99 / 97, at 32 rows
// 101 / 97; 8192 x 8192 at 16 rows 112 / 131, at 32 rows 136 / 132, at 48 rows 150 / 134.
inline bool dense_rows(uint64_t M, uint32_t in_features, uint32_t out_features)
{
    const uint64_t weights = uint64_t(in_features) * out_features;
    if (weights < (1ull << 24)) return M >= 128;
    return M > 64 || (weights >= (1ull << 25) && M > 32 && out_features >= 2 * uint64_t(in_features));
}
inline bool dense_rows_q(uint64_t M, uint32_t in_features, uint32_t out_features)  // quantised codebook
{
    const uint64_t weights = uint64_t(in_features) * out_features;
    if (weights < (1ull << 24)) return M > 64;
    if (weights >= (1ull << 25) && out_features >= 2 * uint64_t(in_features)) return M >= 16;
    return M > 32;
}
// layer_gemm.hip: the weight rebuilt in the register layout of the matrix cores' B operand (layer_weight_frag_bytes
// bytes), the integers of a quantised codebook as a 16-bit codebook for that rebuild, and y [M][out] = x [M][in] . W
// (scale: device pointer or NULL, multiplies the finished sum; partial: layer_gemm_partial_bytes(...) bytes of fp32
// tiles for the tiles whose contraction is cut into slices)
size_t layer_gemm_partial_bytes(uint64_t M, uint32_t in_features, uint32_t out_features);
size_t layer_weight_frag_bytes(uint32_t in_features, uint32_t out_features);
hipError_t launch_layer_weight_frag(const void* codebook, uint32_t K, uint32_t g, const uint16_t* codes, uint32_t in_features,
                                    uint32_t out_features, void* wf, hipStream_t s);
hipError_t launch_codebook_integers16(const void* qbook, int bits, uint32_t K, uint32_t g, int dtype, void* book16, hipStream_t s);
hipError_t launch_layer_gemm(const void* x, uint32_t M, const void* wf, int dtype, uint32_t in_features, uint32_t out_features,
                             const float* scale, const void* bias, void* y, float* partial, hipStream_t s);
// ---- uniformly quantised codebook (layer_quant.hip); bits = 8 or 4
hipError_t launch_codebook_quantize(const float* centroids, size_t n, int bits, void* qbook, float* scale,
                                    uint32_t* absmax_scratch, hipStream_t s);
hipError_t launch_layer_weight_q(const void* qbook, int bits, const float* scale, uint32_t K, uint32_t g,
                                 const uint16_t* codes, uint32_t in_features, uint32_t out_features, int dtype, void* weight,
                                 hipStream_t s);
uint32_t layer_forward_q_max_splits(uint64_t M, uint32_t in_features, uint32_t out_features);
hipError_t launch_layer_forward_q(const void* x, uint32_t M, const void* qbook, int bits, const float* scale, uint32_t K,
                                  uint32_t g, const uint16_t* codes, uint32_t in_features, uint32_t out_features,
                                  const void* bias, void* y, int dtype, float* partial, hipStream_t s);
// grad_weight [in, out] (dtype) -> fp32 vectors [num_codes][d_pad] (zero padding columns and components) and
// codes widened to 32 bits
hipError_t launch_layer_grad_vectors(const void* grad, int dtype, uint32_t in_features, uint32_t out_features,
                                     uint32_t g, uint32_t d_pad, const uint16_t* codes, uint64_t num_codes, float* vectors,
                                     uint32_t* idx, hipStream_t s);

// Diagnostic (probe.hip): the fp16 matrix-core instruction of the E-step on caller-chosen operands.
hipError_t launch_mfma_f16_probe(const uint16_t* A, const uint16_t* B, const float* C, float* D, uint32_t tiles, uint32_t km,
                                 hipStream_t s);

// Reconstruction.
hipError_t launch_decode(const float* C, uint32_t K, uint32_t d, const uint32_t* idx, uint64_t N, float* out,
                         hipStream_t s);

hipError_t launch_copy_f32(const float* src, float* dst, size_t n, hipStream_t s);

// Fixed-point exponent e of the cluster sums: inputs satisfy |x| < 2^(EM+1) with EM the unbiased
// exponent of the largest magnitude M, and N < 2^LN, so |sum of N terms| < 2^(EM+1+e+LN) <= 2^62.
__device__ __forceinline__ int fixed_point_exp(uint32_t absmax_bits, uint32_t N)
{
    const int em = int(absmax_bits >> 23) - 127;   // -127 for zero/subnormal M: fine, just a large e
    const int ln = 32 - __clz(N);                  // N < 2^ln
    const int e = 62 - ln - (em + 1);
    return e < 100 ? e : 100;                      // keep ldexp away from fp64 overflow for tiny inputs
}

// One input as a fixed-point term of the cluster sums. A non-finite input (which the input scan flags in
// WsHeader::x_nonfinite) contributes nothing: its conversion to an integer would be undefined.
__device__ __forceinline__ long long fixed_point_term(float x, int e)
{
    return (__float_as_uint(x) & 0x7f800000u) == 0x7f800000u ? 0ll : __double2ll_rn(ldexp(double(x), e));
}

// Adds (sign = +1) or removes (sign = -1) one vector to/from cluster k's fixed-point sums and count.
// Integer adds commute, so the totals do not depend on the order in which these atomics land.
template <int D>
__device__ __forceinline__ void accumulate_vector(const float (&x)[D], uint32_t k, long long* sums, uint32_t* counts,
                                                  int e, int sign)
{
    unsigned long long* dst = reinterpret_cast<unsigned long long*>(sums + size_t(k) * D);
#pragma unroll
    for (int j = 0; j < D; ++j) {
        const long long f = fixed_point_term(x[j], e);
        if (f != 0) atomicAdd(dst + j, static_cast<unsigned long long>(sign > 0 ? f : -f));
    }
    atomicAdd(counts + k, sign > 0 ? 1u : 0xffffffffu);
}

// ||x - c||^2 in fp32, direct form: first square, then one fused multiply-add per further component.
// Every kernel that needs a distance uses this exact operation order, so that a vector decided by
// one kernel and re-decided by another sees identical values.
template <int D>
__device__ __forceinline__ float direct_sqdist(const float (&x)[D], const float (&c)[D])
{
    const float t0 = x[0] - c[0];
    float acc = t0 * t0;
#pragma unroll
    for (int j = 1; j < D; ++j) {
        const float t = x[j] - c[j];
        acc = __builtin_fmaf(t, t, acc);
    }
    return acc;
}

template <int D>
__device__ __forceinline__ void load_row(const float* __restrict__ p, float (&v)[D]);

// Index recovery of the matrix-core E-step: direct-form argmin over the codebook positions
// 32*(group*GT+g) + 16*h + r, g in [g_begin, g_end), r in [0, 16), of a winning group (the two lanes that
// share a vector split the group's tiles between them). `rows` holds the centroids in packed
// order (the codebook itself, or its norm-ordered copy together with `cperm`, which maps a position
// to the centroid index). Among exactly equal distances the lowest centroid index wins.
// Rows are fetched U at a time so that U independent loads are in flight.
template <int D, int GT>
__device__ __forceinline__ void recover_group(const float (&x)[D], const float* __restrict__ rows,
                                              const uint32_t* __restrict__ cperm, uint32_t K, uint32_t group, int h,
                                              int g_begin, int g_end, float& best_d, uint32_t& best_k)
{
    constexpr int U = D <= 8 ? 8 : 4;
    float bd = INFINITY;
    uint32_t bpos = 0;
    for (int g = g_begin; g < g_end; ++g) {
        const uint32_t k0 = 32 * (group * GT + g) + 16 * h;
#pragma unroll
        for (int r0 = 0; r0 < 16; r0 += U) {
            float c[U][D];
#pragma unroll
            for (int u = 0; u < U; ++u) load_row<D>(rows + size_t(min(k0 + r0 + u, K - 1)) * D, c[u]);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t pos = k0 + r0 + u;
                const float dk = direct_sqdist<D>(x, c[u]);
                if (pos < K) {
                    if (dk < bd) {
                        bd = dk;
                        bpos = pos;
                    } else if (dk == bd && cperm != nullptr && cperm[pos] < cperm[bpos]) {
                        bpos = pos;  // exact tie in norm order: keep the lower centroid index
                    }
                }
            }
        }
    }
    best_d = bd;
    best_k = (cperm != nullptr && bd < INFINITY) ? cperm[min(bpos, K - 1)] : bpos;
}

template <int D>
__device__ __forceinline__ void load_row(const float* __restrict__ p, float (&v)[D])
{
    const float4* s = reinterpret_cast<const float4*>(p);
#pragma unroll
    for (int q = 0; q < D / 4; ++q) {
        const float4 t = s[q];
        v[4 * q + 0] = t.x; v[4 * q + 1] = t.y; v[4 * q + 2] = t.z; v[4 * q + 3] = t.w;
    }
}

}  // namespace cc
