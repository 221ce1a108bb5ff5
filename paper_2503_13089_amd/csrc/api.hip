// C ABI of libcluscomp: argument validation on the host, then the kernel sequence of each call.
// See include/cluscomp.h for the contract of every entry point.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <new>
#include <vector>

#include "../../include/cluscomp.h"
#include "common.h"

namespace {

thread_local char g_err[256] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(hipError_t e, const char* what)
{
    return fail(CC_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int check_shape(uint64_t N, uint32_t d, uint32_t K)
{
    if (d == 0 || d > 16) return fail(CC_ERR_SHAPE, "d = %u is not supported (1..16)", d);
    if (N == 0) return fail(CC_ERR_SHAPE, "N == 0");
    if (N >= (1ull << 32)) return fail(CC_ERR_SHAPE, "N = %llu does not fit 32-bit vector ids", (unsigned long long)N);
    if (K == 0) return fail(CC_ERR_SHAPE, "K == 0");
    if (K > cc::kMaxK) return fail(CC_ERR_SHAPE, "K = %u exceeds the supported maximum %u", K, cc::kMaxK);
    if (K > N) return fail(CC_ERR_SHAPE, "K = %u exceeds N = %llu", K, (unsigned long long)N);
    return CC_OK;
}

int check_layer(uint32_t in_features, uint32_t out_features, uint32_t g, uint32_t K, int dtype, bool allow_f32)
{
    if (in_features == 0 || out_features == 0) return fail(CC_ERR_SHAPE, "in_features == 0 or out_features == 0");
    if (g == 0 || g > 16) return fail(CC_ERR_SHAPE, "g = %u is not supported (1..16)", g);
    if (K == 0 || K > 65536) return fail(CC_ERR_SHAPE, "K = %u does not fit 16-bit codes", K);
    if (!(dtype == CC_F16 || dtype == CC_BF16 || (allow_f32 && dtype == CC_F32)))
        return fail(CC_ERR_SHAPE, "element type %d is not supported here", dtype);
    return CC_OK;
}

int check_workspace(void* ws, size_t ws_bytes, uint64_t N, uint32_t d, uint32_t K)
{
    if (ws == nullptr) return fail(CC_ERR_NULL, "workspace is NULL");
    if (!aligned(ws, 256)) return fail(CC_ERR_ALIGN, "workspace must be 256-byte aligned");
    const size_t need = cc::carve(nullptr, N, d, K).bytes;
    if (ws_bytes < need) return fail(CC_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, need);
    return CC_OK;
}

#define CC_TRY_HIP(expr, what)                        \
    do {                                              \
        hipError_t e_ = (expr);                       \
        if (e_ != hipSuccess) return hip_fail(e_, what); \
    } while (0)

// What one call runs with: the E-step selection (cc_options::assign_mode) and, if the caller asked for device
// times, where they are recorded.
struct Ctx {
    int mode = CC_ASSIGN_AUTO;
    cc::Profile* prof = nullptr;
};

bool use_matrix_cores(const Ctx& cx, uint32_t K)
{
    return cx.mode == CC_ASSIGN_MFMA_F32 || ((cx.mode == CC_ASSIGN_AUTO || cx.mode == CC_ASSIGN_AUTO_WHOLE) && K >= 128);
}

// Norm-window pruning: only in the automatic mode and only where the ordering overhead can pay off. A single
// E-step pays for ordering the vectors by itself, so it needs a large codebook; a fit orders once and keeps the
// integer cluster sums up to date across its iterations, which pays from a few hundred centroids on once there
// are enough vectors to fill the chip (measured break-even: about 3e5 vectors, 5 iterations).
bool use_pruning(const Ctx& cx, uint64_t N, uint32_t K, int32_t iters)
{
    if (cx.mode != CC_ASSIGN_AUTO) return false;
    return K >= 8192 || (K >= 256 && N >= (1u << 19) && iters >= 5);
}

// Relative half-width of the guessed windows of the bootstrap pass. The nearest-centroid distance of a vector of
// norm r is of the order of r * K^(-1/d) when the centroids follow the vectors' own distribution; a window about
// that wide usually holds a near neighbour and is cheap to score. Capped where (large d) no window would be narrow.
float guess_width(uint32_t K, uint32_t d)
{
    const float w = 1.1f * std::pow(float(K), -1.0f / float(d));
    return std::min(0.1f, std::max(0.04f, w));
}

// Scoring + refinement on the matrix cores. The input scan (WsHeader::x_not_f16) must have run on this
// workspace since the last header reset; with pruned = true the vectors must have been norm-ordered
// (launch_sort_vectors) and the codes are left in norm order in w.idx_sorted.
// have_hint = true: the caller knows that this workspace holds the codes of a previous E-step of the same
// call (later iterations of a fit), so the bootstrap pass need not even be enqueued.
int run_assign_matrix(const Ctx& cx, const float* X, uint32_t N, uint32_t d, const float* C, uint32_t K, uint32_t* idx,
                      const cc::Workspace& w, bool accumulate, bool pruned, bool have_hint, hipStream_t s,
                      bool track_changes = false)
{
    const bool both = cx.mode != CC_ASSIGN_MFMA_F32;  // fp16 and fp32 variants enqueued, the device gate picks one
    cc::EStep e{};
    e.profile = cx.prof;
    e.X = pruned ? w.xsorted : X;
    e.N = N;
    e.idx = pruned ? w.idx_sorted : idx;
    if (pruned) {
        {
            cc::ProfileScope order_scope(cx.prof, cc::kProfOrder, s);
            CC_TRY_HIP(cc::launch_sort_centroids(C, d, K, w, s), "assign (centroid norm order)");
        }
        // Bootstrap (only runs on the device when the workspace holds no hint): the nearest centroid inside a
        // guessed window around each vector's own norm and projection. Its codes are only the upper bounds that
        // size the real windows below, so a poor guess costs time, never correctness.
        if (!have_hint) {
            {
                cc::ProfileScope order_scope(cx.prof, cc::kProfOrder, s);
                CC_TRY_HIP(cc::launch_windows(C, N, d, K, w, guess_width(K, d), s), "assign (guessed windows)");
            }
            cc::EStep b = e;
            b.pack_rows = C; b.pack_perm = w.cperm; b.rows = w.csorted; b.row_ids = w.cperm; b.K = K;
            b.packed = w.packed; b.packed_tiles = w.packed_tiles; b.windows = w.windows;
            b.accumulate = false; b.hint_only = true;
            b.gate = cc::kGateIfF16 | cc::kGateNoHint;
            CC_TRY_HIP(cc::launch_assign_mfma_f16(b, d, w, s), "assign (bootstrap, fp16 matrix cores)");
            b.gate = cc::kGateIfNotF16 | cc::kGateNoHint;
            CC_TRY_HIP(cc::launch_assign_mfma_f32(b, d, w, s), "assign (bootstrap, fp32 matrix cores)");
        }
        cc::ProfileScope order_scope(cx.prof, cc::kProfOrder, s);
        CC_TRY_HIP(cc::launch_windows(C, N, d, K, w, 0.0f, s), "assign (norm windows)");
    }
    e.pack_rows = C; e.pack_perm = pruned ? w.cperm : nullptr;
    e.rows = pruned ? w.csorted : C; e.row_ids = pruned ? w.cperm : nullptr;
    e.K = K; e.packed = w.packed; e.packed_tiles = w.packed_tiles;
    e.windows = pruned ? w.windows : nullptr;
    e.accumulate = accumulate; e.hint_only = false;
    // (incremental M-step) the kernel notes which vectors leave the code that e.idx held on entry, and that code
    if (track_changes) { e.prev_out = w.idx_prev; e.changed = w.changed; }
    if (both) {
        e.gate = cc::kGateIfF16;
        CC_TRY_HIP(cc::launch_assign_mfma_f16(e, d, w, s), "assign (fp16 matrix cores)");
        e.gate = cc::kGateIfNotF16;
        CC_TRY_HIP(cc::launch_assign_mfma_f32(e, d, w, s), "assign (fp32 matrix cores)");
    } else {
        e.gate = cc::kGateAlways;
        CC_TRY_HIP(cc::launch_assign_mfma_f32(e, d, w, s), "assign (fp32 matrix cores)");
    }
    {
        cc::ProfileScope refine_scope(cx.prof, cc::kProfRefine, s);
        CC_TRY_HIP(cc::launch_refine(e.X, N, d, C, K, e.idx, w, accumulate, pruned, s), "assign (refinement)");
    }
    return CC_OK;
}

// One E-step pass: idx (and, if inertia != NULL, the objective) for the given centroids.
// to_user = false leaves norm-ordered codes in the workspace only (intermediate fit iterations).
int run_assign(const Ctx& cx, const float* X, uint32_t N, uint32_t d, const float* C, uint32_t K, uint32_t* idx,
               double* inertia, const cc::Workspace& w, bool pruned, bool have_hint, hipStream_t s)
{
    if (use_matrix_cores(cx, K)) {
        if (int rc = run_assign_matrix(cx, X, N, d, C, K, idx, w, false, pruned, have_hint, s)) return rc;
        if (pruned) CC_TRY_HIP(cc::launch_unpermute(N, idx, w, s), "assign (codes to input order)");
    } else {
        CC_TRY_HIP(cc::launch_assign_direct(X, N, d, C, K, idx, w.dmin, nullptr, 0, s, cx.prof), "assign (direct form)");
        CC_TRY_HIP(cc::launch_bump_assign_calls(w.hdr, s), "bookkeeping");
    }
    if (inertia)
        CC_TRY_HIP(cc::launch_reduce_dmin(w.dmin, N, w.partials, w.partial_slots, inertia, s), "objective reduction");
    return CC_OK;
}

// One Lloyd iteration: idx = E-step against C, then C <- M-step(idx) in place. On the matrix-core path
// the cluster sums are accumulated by the scoring kernel itself (no second pass over the vectors).
// idx == NULL (only inside the fit loop, pruned path) skips the copy of the codes to input order.
int run_lloyd_iter(const Ctx& cx, const float* X, uint32_t N, uint32_t d, float* C, uint32_t K, uint32_t* idx,
                   double* inertia, uint32_t* counts, const cc::Workspace& w, bool pruned, bool have_hint, hipStream_t s,
                   bool sums_follow = false)
{
    if (use_matrix_cores(cx, K)) {
        // sums_follow (inside a fit, pruned path, after an M-step by buckets of the same fit): the workspace holds the
        // integer sums and counts of the codes in w.idx_sorted. The E-step kernel then flags the vectors that leave
        // those codes (and keeps the code they had), so that the M-step can move just these.
        // A pruned E-step is shorter than the atomic traffic of the fused accumulation (which then becomes the
        // bottleneck), so there the M-step groups the vectors by bucket of clusters and sums in LDS instead.
        const bool by_buckets = pruned && w.bucket_ok;
        if (!by_buckets) CC_TRY_HIP(cc::launch_zero_accumulators(w, K, d, nullptr, 0, s), "update (clear)");
        if (int rc = run_assign_matrix(cx, X, N, d, C, K, idx, w, !by_buckets, pruned, have_hint, s, sums_follow)) return rc;
        {
            cc::ProfileScope mstep_scope(cx.prof, cc::kProfMstep, s);
            if (by_buckets && !sums_follow && cc::update_sliced_applies(N, d, K, w))
                CC_TRY_HIP(cc::launch_update_sliced(w.xsorted, N, d, w.idx_sorted, C, K, C, counts, w, true, s), "update (slices)");
            else if (by_buckets)
                CC_TRY_HIP(cc::launch_update_buckets(w.xsorted, N, d, w.idx_sorted, C, K, C, counts, w, true, true, s,
                                                     sums_follow ? w.idx_prev : nullptr, sums_follow ? w.changed : nullptr),
                           "update (buckets)");
            else
                CC_TRY_HIP(cc::launch_finalize(C, C, counts, K, d, N, w, true, s), "update (means)");
        }
        if (pruned && idx != nullptr) CC_TRY_HIP(cc::launch_unpermute(N, idx, w, s), "assign (codes to input order)");
    } else {
        CC_TRY_HIP(cc::launch_assign_direct(X, N, d, C, K, idx, w.dmin, nullptr, 0, s, cx.prof), "assign (direct form)");
        CC_TRY_HIP(cc::launch_bump_assign_calls(w.hdr, s), "bookkeeping");
        cc::ProfileScope mstep_scope(cx.prof, cc::kProfMstep, s);
        CC_TRY_HIP(cc::launch_update(X, N, d, idx, C, K, C, counts, w, true, s), "update");
    }
    if (inertia)
        CC_TRY_HIP(cc::launch_reduce_dmin(w.dmin, N, w.partials, w.partial_slots, inertia, s), "objective reduction");
    return CC_OK;
}

// Sub-vector lengths other than 4, 8, 16 run on zero-padded copies (length 4, 8 or 16): padding both the
// vectors and the centroids with zeros changes no distance and no mean. Views of one call's operands:
struct Operands {
    const float* X;       // vectors, rows of w.d floats
    const float* C_in;    // centroids entering the call (NULL if the call has none)
    float* C_work;        // where the kernels read/write centroids
};

int enter(const float* vectors, const float* centroids_in, float* centroids_out, uint32_t N, uint32_t d, uint32_t K,
          const cc::Workspace& w, hipStream_t s, Operands& o)
{
    if (!w.padded) {
        o = {vectors, centroids_in, centroids_out};
        return CC_OK;
    }
    CC_TRY_HIP(cc::launch_pad_rows(vectors, N, d, w.d, w.xpad, s), "padding (vectors)");
    if (centroids_in) CC_TRY_HIP(cc::launch_pad_rows(centroids_in, K, d, w.d, w.cpad, s), "padding (centroids)");
    o = {w.xpad, centroids_in ? w.cpad : nullptr, w.cpad};
    return CC_OK;
}

int leave(float* centroids_out, uint32_t d, uint32_t K, const cc::Workspace& w, hipStream_t s)
{
    if (w.padded && centroids_out) CC_TRY_HIP(cc::launch_unpad_rows(w.cpad, K, w.d, d, centroids_out, s), "padding (result)");
    return CC_OK;
}

// Reads the caller's options (NULL = defaults).
int read_options(const cc_options* o, Ctx& cx)
{
    cx = Ctx{};
    if (o == nullptr) return CC_OK;
    if (o->struct_bytes != sizeof(cc_options))
        return fail(CC_ERR_SHAPE, "cc_options::struct_bytes = %u, this library expects %zu", o->struct_bytes, sizeof(cc_options));
    if (o->assign_mode < CC_ASSIGN_AUTO || o->assign_mode > CC_ASSIGN_AUTO_WHOLE)
        return fail(CC_ERR_SHAPE, "unknown assign mode %d", o->assign_mode);
    cx.mode = o->assign_mode;
    cx.prof = reinterpret_cast<cc::Profile*>(o->profile);
    return CC_OK;
}

}  // namespace

// ---- device-time records (cc_profile) ---------------------------------------------------------------
namespace cc {

struct Profile {
    struct Record {
        int slot;
        hipEvent_t start, stop;
    };
    std::vector<Record> records;  // events created once, by cc_profile_create
    uint32_t used = 0;
    uint32_t dropped = 0;
    uint32_t mask = 0;
};

ProfileScope::ProfileScope(Profile* p, int slot, hipStream_t s) : p_(p), s_(s), record_(-1)
{
    if (p == nullptr || !(p->mask & (1u << slot))) return;
    if (p->used >= p->records.size()) {
        ++p->dropped;
        return;
    }
    record_ = int(p->used++);
    p->records[record_].slot = slot;
    (void)hipEventRecord(p->records[record_].start, s);
}

ProfileScope::~ProfileScope()
{
    if (record_ >= 0) (void)hipEventRecord(p_->records[record_].stop, s_);
}

}  // namespace cc

extern "C" {

int cc_profile_create(uint32_t max_records, uint32_t slot_mask, cc_profile** out)
{
    if (out == nullptr) return fail(CC_ERR_NULL, "out is NULL");
    *out = nullptr;
    if (max_records == 0 || max_records > 65536) return fail(CC_ERR_SHAPE, "max_records = %u is not in 1..65536", max_records);
    if (slot_mask == 0 || slot_mask >= (1u << CC_PROF_SLOTS)) return fail(CC_ERR_SHAPE, "slot_mask = 0x%x names no known slot", slot_mask);
    cc::Profile* p = new (std::nothrow) cc::Profile;
    if (p == nullptr) return fail(CC_ERR_HIP, "out of host memory");
    p->mask = slot_mask;
    p->records.reserve(max_records);
    for (uint32_t i = 0; i < max_records; ++i) {
        cc::Profile::Record r{};
        hipError_t e = hipEventCreate(&r.start);
        if (e == hipSuccess) {
            e = hipEventCreate(&r.stop);
            if (e != hipSuccess) (void)hipEventDestroy(r.start);
        }
        if (e != hipSuccess) {
            cc_profile_destroy(reinterpret_cast<cc_profile*>(p));
            return hip_fail(e, "event creation");
        }
        p->records.push_back(r);
    }
    *out = reinterpret_cast<cc_profile*>(p);
    return CC_OK;
}

int cc_profile_read(cc_profile* profile, double* ms, uint32_t* launches, uint32_t* dropped)
{
    if (profile == nullptr || ms == nullptr || launches == nullptr) return fail(CC_ERR_NULL, "a required pointer is NULL");
    cc::Profile* p = reinterpret_cast<cc::Profile*>(profile);
    for (int k = 0; k < CC_PROF_SLOTS; ++k) {
        ms[k] = 0.0;
        launches[k] = 0;
    }
    int rc = CC_OK;
    for (uint32_t i = 0; i < p->used; ++i) {
        const cc::Profile::Record& r = p->records[i];
        float t = 0.0f;
        hipError_t e = hipEventSynchronize(r.stop);
        if (e == hipSuccess) e = hipEventElapsedTime(&t, r.start, r.stop);
        if (e != hipSuccess) {
            rc = hip_fail(e, "event read");
            continue;
        }
        ms[r.slot] += double(t);
        launches[r.slot] += 1;
    }
    if (dropped) *dropped = p->dropped;
    p->used = 0;
    p->dropped = 0;
    return rc;
}

void cc_profile_destroy(cc_profile* profile)
{
    cc::Profile* p = reinterpret_cast<cc::Profile*>(profile);
    if (p == nullptr) return;
    for (auto& r : p->records) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    delete p;
}

size_t cc_workspace_bytes(uint64_t N, uint32_t d, uint32_t K)
{
    if (check_shape(N, d, K) != CC_OK) return 0;
    return cc::carve(nullptr, N, d, K).bytes;
}

int cc_kmeans_fit(const float* vectors, uint64_t N, uint32_t d, uint32_t K, int32_t iters, const float* init_centroids,
                  float* centroids, uint32_t* idx, double* inertia, void* workspace, size_t workspace_bytes,
                  void* stream)
{
    return cc_kmeans_fit_ex(vectors, N, d, K, iters, init_centroids, centroids, idx, inertia, workspace, workspace_bytes,
                            stream, nullptr);
}

int cc_kmeans_fit_ex(const float* vectors, uint64_t N, uint32_t d, uint32_t K, int32_t iters, const float* init_centroids,
                     float* centroids, uint32_t* idx, double* inertia, void* workspace, size_t workspace_bytes,
                     void* stream, const cc_options* options)
{
    Ctx cx;
    if (int rc = read_options(options, cx)) return rc;
    if (!vectors || !init_centroids || !centroids || !idx) return fail(CC_ERR_NULL, "a required pointer is NULL");
    if (int rc = check_shape(N, d, K)) return rc;
    if (iters < 0) return fail(CC_ERR_ITERS, "iters = %d is negative", iters);
    if (!aligned(vectors, 16) || !aligned(init_centroids, 16) || !aligned(centroids, 16) || !aligned(idx, 4) ||
        (inertia && !aligned(inertia, 8)))
        return fail(CC_ERR_ALIGN, "vectors/centroids need 16-byte alignment, idx 4, inertia 8");
    if (int rc = check_workspace(workspace, workspace_bytes, N, d, K)) return rc;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const cc::Workspace w = cc::carve(workspace, N, d, K);
    const uint32_t n = uint32_t(N), D = w.d;

    CC_TRY_HIP(cc::launch_reset_header(w.hdr, s), "bookkeeping");
    Operands o;
    if (int rc = enter(vectors, init_centroids, centroids, n, d, K, w, s, o)) return rc;
    CC_TRY_HIP(cc::launch_scan_inputs(o.X, N * D, w.hdr, s), "input scan");
    if (o.C_work != o.C_in)
        CC_TRY_HIP(cc::launch_copy_f32(o.C_in, o.C_work, size_t(K) * D, s), "centroid copy");
    const bool pruned = use_matrix_cores(cx, K) && use_pruning(cx, N, K, iters);
    if (pruned) {
        cc::ProfileScope order_scope(cx.prof, cc::kProfOrder, s);
        CC_TRY_HIP(cc::launch_sort_vectors(o.X, n, D, K, w, true, s), "norm ordering");
    }
    for (int32_t t = 0; t < iters; ++t) {
        // only the matrix-core path can leave its codes in the workspace; the others write idx directly
        uint32_t* step_idx = pruned ? nullptr : idx;
        // from the third iteration on the M-step only moves the vectors whose code changed (the first iterations move
        // too many for that to pay off)
        const bool sums_follow = pruned && w.bucket_ok && t >= 2;
        if (int rc = run_lloyd_iter(cx, o.X, n, D, o.C_work, K, step_idx, nullptr, nullptr, w, pruned, t > 0, s, sums_follow))
            return rc;
    }
    if (int rc = run_assign(cx, o.X, n, D, o.C_work, K, idx, inertia, w, pruned, iters > 0, s)) return rc;
    return leave(centroids, d, K, w, s);
}

int cc_assign(const float* vectors, uint64_t N, uint32_t d, const float* centroids, uint32_t K, uint32_t* idx,
              double* inertia, void* workspace, size_t workspace_bytes, void* stream)
{
    return cc_assign_ex(vectors, N, d, centroids, K, idx, inertia, workspace, workspace_bytes, stream, nullptr);
}

int cc_assign_ex(const float* vectors, uint64_t N, uint32_t d, const float* centroids, uint32_t K, uint32_t* idx,
                 double* inertia, void* workspace, size_t workspace_bytes, void* stream, const cc_options* options)
{
    Ctx cx;
    if (int rc = read_options(options, cx)) return rc;
    if (!vectors || !centroids || !idx) return fail(CC_ERR_NULL, "a required pointer is NULL");
    if (int rc = check_shape(N, d, K)) return rc;
    if (!aligned(vectors, 16) || !aligned(centroids, 16) || !aligned(idx, 4) || (inertia && !aligned(inertia, 8)))
        return fail(CC_ERR_ALIGN, "vectors/centroids need 16-byte alignment, idx 4, inertia 8");
    if (int rc = check_workspace(workspace, workspace_bytes, N, d, K)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const cc::Workspace w = cc::carve(workspace, N, d, K);
    CC_TRY_HIP(cc::launch_reset_header(w.hdr, s), "bookkeeping");
    Operands o;
    if (int rc = enter(vectors, centroids, nullptr, uint32_t(N), d, K, w, s, o)) return rc;
    CC_TRY_HIP(cc::launch_scan_inputs(o.X, N * w.d, w.hdr, s), "input scan");
    const bool pruned = use_matrix_cores(cx, K) && use_pruning(cx, N, K, 1);
    if (pruned) {
        cc::ProfileScope order_scope(cx.prof, cc::kProfOrder, s);
        CC_TRY_HIP(cc::launch_sort_vectors(o.X, uint32_t(N), w.d, K, w, false, s), "norm ordering");
    }
    return run_assign(cx, o.X, uint32_t(N), w.d, o.C_in, K, idx, inertia, w, pruned, false, s);
}

int cc_lloyd_iter(const float* vectors, uint64_t N, uint32_t d, float* centroids, uint32_t K, uint32_t* idx,
                  double* inertia, uint32_t* counts, void* workspace, size_t workspace_bytes, void* stream)
{
    return cc_lloyd_iter_ex(vectors, N, d, centroids, K, idx, inertia, counts, workspace, workspace_bytes, stream, nullptr);
}

int cc_lloyd_iter_ex(const float* vectors, uint64_t N, uint32_t d, float* centroids, uint32_t K, uint32_t* idx,
                     double* inertia, uint32_t* counts, void* workspace, size_t workspace_bytes, void* stream,
                     const cc_options* options)
{
    Ctx cx;
    if (int rc = read_options(options, cx)) return rc;
    if (!vectors || !centroids || !idx) return fail(CC_ERR_NULL, "a required pointer is NULL");
    if (int rc = check_shape(N, d, K)) return rc;
    if (!aligned(vectors, 16) || !aligned(centroids, 16) || !aligned(idx, 4) || (inertia && !aligned(inertia, 8)) ||
        (counts && !aligned(counts, 4)))
        return fail(CC_ERR_ALIGN, "vectors/centroids need 16-byte alignment, idx and counts 4, inertia 8");
    if (int rc = check_workspace(workspace, workspace_bytes, N, d, K)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const cc::Workspace w = cc::carve(workspace, N, d, K);
    CC_TRY_HIP(cc::launch_reset_header(w.hdr, s), "bookkeeping");
    Operands o;
    if (int rc = enter(vectors, centroids, centroids, uint32_t(N), d, K, w, s, o)) return rc;
    CC_TRY_HIP(cc::launch_scan_inputs(o.X, N * w.d, w.hdr, s), "input scan");
    const bool pruned = use_matrix_cores(cx, K) && use_pruning(cx, N, K, 1);
    if (pruned) {
        cc::ProfileScope order_scope(cx.prof, cc::kProfOrder, s);
        CC_TRY_HIP(cc::launch_sort_vectors(o.X, uint32_t(N), w.d, K, w, false, s), "norm ordering");
    }
    if (int rc = run_lloyd_iter(cx, o.X, uint32_t(N), w.d, o.C_work, K, idx, inertia, counts, w, pruned, false, s)) return rc;
    return leave(centroids, d, K, w, s);
}

int cc_update(const float* vectors, uint64_t N, uint32_t d, const uint32_t* idx, const float* prev_centroids,
              uint32_t K, float* centroids, uint32_t* counts, void* workspace, size_t workspace_bytes, void* stream)
{
    return cc_update_ex(vectors, N, d, idx, prev_centroids, K, centroids, counts, workspace, workspace_bytes, stream, nullptr);
}

int cc_update_ex(const float* vectors, uint64_t N, uint32_t d, const uint32_t* idx, const float* prev_centroids,
                 uint32_t K, float* centroids, uint32_t* counts, void* workspace, size_t workspace_bytes, void* stream,
                 const cc_options* options)
{
    Ctx cx;
    if (int rc = read_options(options, cx)) return rc;
    if (!vectors || !idx || !prev_centroids || !centroids) return fail(CC_ERR_NULL, "a required pointer is NULL");
    if (int rc = check_shape(N, d, K)) return rc;
    if (!aligned(vectors, 16) || !aligned(prev_centroids, 16) || !aligned(centroids, 16) || !aligned(idx, 4) ||
        (counts && !aligned(counts, 4)))
        return fail(CC_ERR_ALIGN, "vectors/centroids need 16-byte alignment, idx and counts 4");
    if (int rc = check_workspace(workspace, workspace_bytes, N, d, K)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const cc::Workspace w = cc::carve(workspace, N, d, K);
    CC_TRY_HIP(cc::launch_reset_header(w.hdr, s), "bookkeeping");
    Operands o;
    if (int rc = enter(vectors, prev_centroids, centroids, uint32_t(N), d, K, w, s, o)) return rc;
    CC_TRY_HIP(cc::launch_scan_inputs(o.X, N * w.d, w.hdr, s), "input scan");
    {
        cc::ProfileScope mstep_scope(cx.prof, cc::kProfMstep, s);
        CC_TRY_HIP(cc::launch_update(o.X, uint32_t(N), w.d, idx, o.C_in, K, o.C_work, counts, w, true, s), "update");
    }
    return leave(centroids, d, K, w, s);
}

int cc_decode(const float* centroids, uint32_t K, uint32_t d, const uint32_t* idx, uint64_t N, float* out,
              void* stream)
{
    if (!centroids || !idx || !out) return fail(CC_ERR_NULL, "a required pointer is NULL");
    if (d == 0 || d > 16) return fail(CC_ERR_SHAPE, "d = %u is not supported (1..16)", d);
    if (N == 0 || K == 0) return fail(CC_ERR_SHAPE, "N == 0 or K == 0");
    if (N >= (1ull << 32)) return fail(CC_ERR_SHAPE, "N = %llu does not fit 32-bit vector ids", (unsigned long long)N);
    if (!aligned(centroids, 16) || !aligned(out, 16) || !aligned(idx, 4))
        return fail(CC_ERR_ALIGN, "centroids/out need 16-byte alignment, idx 4");
    CC_TRY_HIP(cc::launch_decode(centroids, K, d, idx, N, out, static_cast<hipStream_t>(stream)), "decode");
    return CC_OK;
}

// ---- the compressed linear layer -----------------------------------------------------------------

uint32_t cc_layer_deficiency(uint32_t out_features, uint32_t g)
{
    if (g == 0) return 0;
    const uint32_t r = out_features % g;
    return r == 0 ? 0 : g - r;
}

uint64_t cc_layer_num_codes(uint64_t in_features, uint64_t out_features, uint32_t g)
{
    if (g == 0) return 0;
    return in_features * ((out_features + g - 1) / g);
}

int cc_layer_vectors(const void* weight, int weight_dtype, uint32_t out_features, uint32_t in_features, uint32_t g,
                     float* vectors, void* stream)
{
    if (!weight || !vectors) return fail(CC_ERR_NULL, "a required pointer is NULL");
    if (int rc = check_layer(in_features, out_features, g, 1, weight_dtype, true)) return rc;
    if (!aligned(weight, 4) || !aligned(vectors, 16)) return fail(CC_ERR_ALIGN, "vectors need 16-byte alignment");
    CC_TRY_HIP(cc::launch_layer_vectors(weight, weight_dtype, out_features, in_features, g, vectors,
                                        static_cast<hipStream_t>(stream)), "layer vectors");
    return CC_OK;
}

int cc_layer_pack(const float* centroids, uint32_t K, uint32_t g, void* codebook, int codebook_dtype,
                  const uint32_t* idx, uint64_t num_codes, uint16_t* codes, void* stream)
{
    if ((centroids == nullptr) != (codebook == nullptr) || (idx == nullptr) != (codes == nullptr) ||
        (centroids == nullptr && idx == nullptr))
        return fail(CC_ERR_NULL, "pass both pointers of at least one of the pairs (centroids, codebook), (idx, codes)");
    if (K == 0 || K > 65536) return fail(CC_ERR_SHAPE, "K = %u does not fit 16-bit codes", K);
    if (g == 0 || g > 16) return fail(CC_ERR_SHAPE, "g = %u is not supported (1..16)", g);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (centroids) {
        if (codebook_dtype != CC_F16 && codebook_dtype != CC_BF16)
            return fail(CC_ERR_SHAPE, "the stored codebook is CC_F16 or CC_BF16");
        if (!aligned(centroids, 4) || !aligned(codebook, 2)) return fail(CC_ERR_ALIGN, "misaligned codebook");
        CC_TRY_HIP(cc::launch_layer_pack_codebook(centroids, size_t(K) * g, codebook, codebook_dtype, s), "codebook format");
    }
    if (idx) {
        if (num_codes == 0 || num_codes >= (1ull << 32)) return fail(CC_ERR_SHAPE, "num_codes = %llu", (unsigned long long)num_codes);
        if (!aligned(idx, 4) || !aligned(codes, 2)) return fail(CC_ERR_ALIGN, "misaligned codes");
        CC_TRY_HIP(cc::launch_layer_pack_codes(idx, num_codes, K, codes, s), "code format");
    }
    return CC_OK;
}

int cc_layer_weight(const void* codebook, int dtype, uint32_t K, uint32_t g, const uint16_t* codes,
                    uint32_t in_features, uint32_t out_features, void* weight, void* stream)
{
    if (!codebook || !codes || !weight) return fail(CC_ERR_NULL, "a required pointer is NULL");
    if (int rc = check_layer(in_features, out_features, g, K, dtype, true)) return rc;
    if (!aligned(codebook, 16) || !aligned(weight, 16) || !aligned(codes, 2))
        return fail(CC_ERR_ALIGN, "codebook/weight need 16-byte alignment, codes 2");
    CC_TRY_HIP(cc::launch_layer_weight(codebook, dtype, K, g, codes, in_features, out_features, weight,
                                       static_cast<hipStream_t>(stream)), "layer weight");
    return CC_OK;
}

size_t cc_layer_forward_workspace_bytes(uint64_t M, uint32_t in_features, uint32_t out_features)
{
    if (M == 0 || M > (1ull << 22) || in_features == 0 || out_features == 0) return 0;
    uint32_t splits = cc::layer_forward_splits(M, in_features, out_features);
    // the sub-vector length is not an argument here: few rows of x may take the kernel with the finer slices
    if (cc::layer_forward_few_rows(M, 4)) splits = std::max(splits, cc::layer_forward_few_rows_max_splits());
    const size_t fused = splits > 1 ? cc::align256(size_t(splits) * M * out_features * 4) : 0;
    if (!cc::dense_rows(M, in_features, out_features)) return fused;
    // the rebuilt 16-bit weight (matrix-core operand layout), then the fp32 partial tiles of a contraction split over
    // workgroups
    return cc::layer_weight_frag_bytes(in_features, out_features) + cc::layer_gemm_partial_bytes(M, in_features, out_features);
}

int cc_layer_forward(const void* x, uint64_t M, const void* codebook, int dtype, uint32_t K, uint32_t g,
                     const uint16_t* codes, uint32_t in_features, uint32_t out_features, const void* bias, void* y,
                     void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !codebook || !codes || !y) return fail(CC_ERR_NULL, "a required pointer is NULL");
    if (int rc = check_layer(in_features, out_features, g, K, dtype, false)) return rc;
    if (M == 0 || M > (1ull << 22)) return fail(CC_ERR_SHAPE, "M = %llu is not in 1..2^22", (unsigned long long)M);
    if (in_features % 8 != 0) return fail(CC_ERR_SHAPE, "in_features = %u is not a multiple of 8", in_features);
    if (!aligned(x, 16) || !aligned(y, 16) || !aligned(codebook, 16) || !aligned(codes, 2) || (bias && !aligned(bias, 2)))
        return fail(CC_ERR_ALIGN, "x, y and codebook need 16-byte alignment");
    const size_t need = cc_layer_forward_workspace_bytes(M, in_features, out_features);
    if (need > 0) {
        if (workspace == nullptr) return fail(CC_ERR_NULL, "workspace is NULL");
        if (!aligned(workspace, 256)) return fail(CC_ERR_ALIGN, "workspace must be 256-byte aligned");
        if (workspace_bytes < need) return fail(CC_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (cc::dense_rows(M, in_features, out_features)) {
        char* partial = static_cast<char*>(workspace) + cc::layer_weight_frag_bytes(in_features, out_features);
        CC_TRY_HIP(cc::launch_layer_weight_frag(codebook, K, g, codes, in_features, out_features, workspace, s), "layer weight");
        CC_TRY_HIP(cc::launch_layer_gemm(x, uint32_t(M), workspace, dtype, in_features, out_features, nullptr, bias, y,
                                         reinterpret_cast<float*>(partial), s), "dense product");
        return CC_OK;
    }
    CC_TRY_HIP(cc::launch_layer_forward(x, uint32_t(M), codebook, dtype, K, g, codes, in_features, out_features, bias, y,
                                        static_cast<float*>(workspace), s), "layer forward");
    return CC_OK;
}

int cc_layer_codebook_grad(const void* grad_weight, int grad_dtype, uint32_t in_features, uint32_t out_features,
                           const uint16_t* codes, uint32_t K, uint32_t g, float* grad_codebook, void* workspace,
                           size_t workspace_bytes, void* stream)
{
    if (!grad_weight || !codes || !grad_codebook) return fail(CC_ERR_NULL, "a required pointer is NULL");
    if (int rc = check_layer(in_features, out_features, g, K, grad_dtype, true)) return rc;
    const uint64_t N = cc_layer_num_codes(in_features, out_features, g);
    if (N >= (1ull << 32)) return fail(CC_ERR_SHAPE, "num_codes = %llu does not fit 32-bit vector ids", (unsigned long long)N);
    if (!aligned(grad_weight, 4) || !aligned(grad_codebook, 16) || !aligned(codes, 2))
        return fail(CC_ERR_ALIGN, "grad_codebook needs 16-byte alignment, grad_weight 4, codes 2");
    if (workspace == nullptr) return fail(CC_ERR_NULL, "workspace is NULL");
    if (!aligned(workspace, 256)) return fail(CC_ERR_ALIGN, "workspace must be 256-byte aligned");
    // sized like a clustering problem with at least K vectors (a layer may have fewer codes than clusters)
    const uint64_t n_ws = N > K ? N : K;
    const size_t need = cc::carve(nullptr, n_ws, g, K).bytes;
    if (workspace_bytes < need) return fail(CC_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const cc::Workspace w = cc::carve(workspace, n_ws, g, K);
    CC_TRY_HIP(cc::launch_reset_header(w.hdr, s), "bookkeeping");
    // A large layer with 16-bit gradients whose sub-vectors are whole rows of g numbers: summed in place by cluster
    // slices, no fp32 copy of the gradient (the same fixed-point sums as below, hence the same bits).
    if (grad_dtype != CC_F32 && out_features % g == 0 && !w.padded && aligned(grad_weight, 16) && aligned(codes, 4) &&
        cc::update_sliced_applies(uint32_t(N), w.d, K, w)) {
        CC_TRY_HIP(cc::launch_scan_inputs16(grad_weight, grad_dtype, N * g, w.hdr, s), "input scan");
        CC_TRY_HIP(cc::launch_sum_rows16_sliced(grad_weight, grad_dtype, uint32_t(N), w.d, codes, K, grad_codebook, w, s),
                   "codebook gradient (slices)");
        return CC_OK;
    }
    // the ordered-copy buffers of the E-step are free here: vectors in w.xsorted, widened codes in w.idx_sorted
    CC_TRY_HIP(cc::launch_layer_grad_vectors(grad_weight, grad_dtype, in_features, out_features, g, w.d, codes, N, w.xsorted,
                                             w.idx_sorted, s), "gradient vectors");
    CC_TRY_HIP(cc::launch_scan_inputs(w.xsorted, N * w.d, w.hdr, s), "input scan");
    float* out = w.padded ? w.csorted : grad_codebook;
    CC_TRY_HIP(cc::launch_update(w.xsorted, uint32_t(N), w.d, w.idx_sorted, nullptr, K, out, nullptr, w, false, s),
               "codebook gradient");
    if (w.padded) CC_TRY_HIP(cc::launch_unpad_rows(w.csorted, K, w.d, g, grad_codebook, s), "padding (result)");
    return CC_OK;
}

// One layer, one call: reshape, seeded start, Lloyd iterations, storage formats.
namespace {
struct CompressLayout {
    size_t vectors, centroids, idx, fit, total;
    uint64_t N;
};
CompressLayout compress_layout(uint32_t out_features, uint32_t in_features, uint32_t g, uint32_t K)
{
    CompressLayout l{};
    l.N = cc_layer_num_codes(in_features, out_features, g);
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t at = off; off += cc::align256(bytes); return at; };
    l.vectors = take(size_t(l.N) * g * 4);
    l.centroids = take(size_t(K) * g * 4);
    l.idx = take(size_t(l.N) * 4);
    l.fit = take(cc::carve(nullptr, l.N, g, K).bytes);
    l.total = off;
    return l;
}
}  // namespace

size_t cc_layer_compress_workspace_bytes(uint32_t out_features, uint32_t in_features, uint32_t g, uint32_t K)
{
    if (check_layer(in_features, out_features, g, K, CC_BF16, true) != CC_OK) return 0;
    const CompressLayout l = compress_layout(out_features, in_features, g, K);
    if (check_shape(l.N, g, K) != CC_OK) return 0;
    return l.total;
}

int cc_layer_compress(const void* weight, int weight_dtype, uint32_t out_features, uint32_t in_features, uint32_t g,
                      uint32_t K, int32_t iters, const uint32_t* init_ids, void* codebook, int codebook_dtype,
                      uint16_t* codes, double* inertia, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!weight || !init_ids || !codebook || !codes) return fail(CC_ERR_NULL, "a required pointer is NULL");
    if (int rc = check_layer(in_features, out_features, g, K, weight_dtype, true)) return rc;
    if (codebook_dtype != CC_F16 && codebook_dtype != CC_BF16) return fail(CC_ERR_SHAPE, "the stored codebook is CC_F16 or CC_BF16");
    if (iters < 0) return fail(CC_ERR_ITERS, "iters = %d is negative", iters);
    const CompressLayout l = compress_layout(out_features, in_features, g, K);
    if (int rc = check_shape(l.N, g, K)) return rc;
    if (workspace == nullptr) return fail(CC_ERR_NULL, "workspace is NULL");
    if (!aligned(workspace, 256)) return fail(CC_ERR_ALIGN, "workspace must be 256-byte aligned");
    if (workspace_bytes < l.total) return fail(CC_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, l.total);
    char* base = static_cast<char*>(workspace);
    float* vectors = reinterpret_cast<float*>(base + l.vectors);
    float* centroids = reinterpret_cast<float*>(base + l.centroids);
    uint32_t* idx = reinterpret_cast<uint32_t*>(base + l.idx);
    if (int rc = cc_layer_vectors(weight, weight_dtype, out_features, in_features, g, vectors, stream)) return rc;
    // the starting centroids are the listed vectors: a gather of rows, i.e. a decode with the vectors as the table
    if (int rc = cc_decode(vectors, uint32_t(l.N), g, init_ids, K, centroids, stream)) return rc;
    if (int rc = cc_kmeans_fit(vectors, l.N, g, K, iters, centroids, centroids, idx, inertia, base + l.fit,
                               workspace_bytes - l.fit, stream))
        return rc;
    return cc_layer_pack(centroids, K, g, codebook, codebook_dtype, idx, l.N, codes, stream);
}

// ---- uniformly quantised codebook ---------------------------------------------------------------

int cc_codebook_quantize(const float* centroids, uint32_t K, uint32_t g, int bits, void* qbook, float* scale,
                         void* scratch, void* stream)
{
    if (!centroids || !qbook || !scale || !scratch) return fail(CC_ERR_NULL, "a required pointer is NULL");
    if (K == 0 || K > 65536) return fail(CC_ERR_SHAPE, "K = %u does not fit 16-bit codes", K);
    if (g == 0 || g > 16) return fail(CC_ERR_SHAPE, "g = %u is not supported (1..16)", g);
    if (bits != 8 && bits != 4) return fail(CC_ERR_SHAPE, "bits = %d is not supported (8, 4)", bits);
    if (!aligned(centroids, 4) || !aligned(scale, 4) || !aligned(scratch, 4)) return fail(CC_ERR_ALIGN, "misaligned pointer");
    CC_TRY_HIP(cc::launch_codebook_quantize(centroids, size_t(K) * g, bits, qbook, scale, static_cast<uint32_t*>(scratch),
                                            static_cast<hipStream_t>(stream)), "codebook quantisation");
    return CC_OK;
}

int cc_layer_weight_q(const void* qbook, int bits, const float* scale, uint32_t K, uint32_t g, const uint16_t* codes,
                      uint32_t in_features, uint32_t out_features, int dtype, void* weight, void* stream)
{
    if (!qbook || !scale || !codes || !weight) return fail(CC_ERR_NULL, "a required pointer is NULL");
    if (int rc = check_layer(in_features, out_features, g, K, dtype, false)) return rc;
    if (bits != 8 && bits != 4) return fail(CC_ERR_SHAPE, "bits = %d is not supported (8, 4)", bits);
    if (!aligned(qbook, 16) || !aligned(weight, 16) || !aligned(codes, 2) || !aligned(scale, 4))
        return fail(CC_ERR_ALIGN, "qbook/weight need 16-byte alignment, codes 2, scale 4");
    CC_TRY_HIP(cc::launch_layer_weight_q(qbook, bits, scale, K, g, codes, in_features, out_features, dtype, weight,
                                         static_cast<hipStream_t>(stream)), "layer weight (quantised codebook)");
    return CC_OK;
}

size_t cc_layer_grad_plan_bytes(uint64_t num_codes, uint32_t K)
{
    if (num_codes == 0 || num_codes >= (1ull << 32) || K == 0 || K > 65536) return 0;
    return cc::layer_grad_plan_bytes(num_codes, K);
}

size_t cc_layer_grad_plan_workspace_bytes(uint64_t num_codes)
{
    if (num_codes == 0 || num_codes >= (1ull << 32)) return 0;
    return cc::layer_grad_plan_build_bytes(num_codes);
}

int cc_layer_grad_plan(const uint16_t* codes, uint64_t num_codes, uint32_t K, void* plan, size_t plan_bytes, void* workspace,
                       size_t workspace_bytes, void* stream)
{
    if (!codes || !plan || !workspace) return fail(CC_ERR_NULL, "a required pointer is NULL");
    if (num_codes == 0 || num_codes >= (1ull << 32)) return fail(CC_ERR_SHAPE, "num_codes = %llu", (unsigned long long)num_codes);
    if (K == 0 || K > 65536) return fail(CC_ERR_SHAPE, "K = %u is not in 1..65536", K);
    if (!aligned(codes, 2) || !aligned(plan, 256) || !aligned(workspace, 256))
        return fail(CC_ERR_ALIGN, "plan and workspace must be 256-byte aligned, codes 2");
    if (plan_bytes < cc::layer_grad_plan_bytes(num_codes, K))
        return fail(CC_ERR_WORKSPACE, "plan has %zu bytes, %zu needed", plan_bytes, cc::layer_grad_plan_bytes(num_codes, K));
    if (workspace_bytes < cc::layer_grad_plan_build_bytes(num_codes))
        return fail(CC_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes,
                    cc::layer_grad_plan_build_bytes(num_codes));
    CC_TRY_HIP(cc::launch_layer_grad_plan(codes, uint32_t(num_codes), K, plan, workspace, static_cast<hipStream_t>(stream)),
               "gradient plan");
    return CC_OK;
}

size_t cc_layer_codebook_grad_planned_workspace_bytes(uint64_t num_codes, uint32_t K, uint32_t g)
{
    if (num_codes == 0 || num_codes >= (1ull << 32) || K == 0 || K > 65536 || g == 0 || g > 16) return 0;
    return cc::layer_grad_planned_bytes(num_codes, K, g);
}

int cc_layer_codebook_grad_planned(const void* grad_weight, int grad_dtype, uint32_t in_features, uint32_t out_features,
                                   uint32_t K, uint32_t g, const void* plan, size_t plan_bytes, float* grad_codebook,
                                   void* workspace, size_t workspace_bytes, void* stream)
{
    if (!grad_weight || !plan || !grad_codebook || !workspace) return fail(CC_ERR_NULL, "a required pointer is NULL");
    if (int rc = check_layer(in_features, out_features, g, K, grad_dtype, true)) return rc;
    const uint64_t N = cc_layer_num_codes(in_features, out_features, g);
    if (N >= (1ull << 32)) return fail(CC_ERR_SHAPE, "num_codes = %llu does not fit 32-bit positions", (unsigned long long)N);
    if (!aligned(grad_weight, 16) || !aligned(grad_codebook, 4) || !aligned(plan, 256) || !aligned(workspace, 256))
        return fail(CC_ERR_ALIGN, "grad_weight needs 16-byte alignment, plan and workspace 256");
    if (plan_bytes < cc::layer_grad_plan_bytes(N, K))
        return fail(CC_ERR_WORKSPACE, "plan has %zu bytes, %zu needed for these shapes", plan_bytes, cc::layer_grad_plan_bytes(N, K));
    const size_t need = cc::layer_grad_planned_bytes(N, K, g);
    if (workspace_bytes < need) return fail(CC_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
    CC_TRY_HIP(cc::launch_layer_grad_planned(grad_weight, grad_dtype, in_features, out_features, K, g, uint32_t(N), plan,
                                             grad_codebook, workspace, static_cast<hipStream_t>(stream)),
               "codebook gradient (planned)");
    return CC_OK;
}

namespace {
constexpr size_t kIntegerBookBytes = size_t(65536) * 16 * 2;  // K <= 65536 codes of g <= 16 entries, 16 bits each
}

size_t cc_layer_forward_q_workspace_bytes(uint64_t M, uint32_t in_features, uint32_t out_features)
{
    if (M == 0 || M > (1ull << 22) || in_features == 0 || out_features == 0) return 0;
    const uint32_t splits = cc::layer_forward_q_max_splits(M, in_features, out_features);
    const size_t fused = splits > 1 ? cc::align256(size_t(splits) * M * out_features * 4) : 0;
    if (!cc::dense_rows_q(M, in_features, out_features)) return fused;
    // the integer weight in 16 bits (matrix-core operand layout), the integer codebook in 16 bits (at most 65536 x 16
    // entries), then the fp32 partial tiles of the product
    const size_t dense = cc::layer_weight_frag_bytes(in_features, out_features) + kIntegerBookBytes +
                         cc::layer_gemm_partial_bytes(M, in_features, out_features);
    return dense > fused ? dense : fused;
}

int cc_layer_forward_q(const void* x, uint64_t M, const void* qbook, int bits, const float* scale, uint32_t K, uint32_t g,
                       const uint16_t* codes, uint32_t in_features, uint32_t out_features, const void* bias, void* y,
                       int dtype, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !qbook || !scale || !codes || !y) return fail(CC_ERR_NULL, "a required pointer is NULL");
    if (int rc = check_layer(in_features, out_features, g, K, dtype, false)) return rc;
    if (bits != 8 && bits != 4) return fail(CC_ERR_SHAPE, "bits = %d is not supported (8, 4)", bits);
    if (M == 0 || M > (1ull << 22)) return fail(CC_ERR_SHAPE, "M = %llu is not in 1..2^22", (unsigned long long)M);
    if (in_features % 8 != 0) return fail(CC_ERR_SHAPE, "in_features = %u is not a multiple of 8", in_features);
    if (!aligned(x, 16) || !aligned(y, 16) || !aligned(qbook, 16) || !aligned(codes, 2) || !aligned(scale, 4) ||
        (bias && !aligned(bias, 2)))
        return fail(CC_ERR_ALIGN, "x, y and qbook need 16-byte alignment");
    const size_t need = cc_layer_forward_q_workspace_bytes(M, in_features, out_features);
    if (need > 0) {
        if (workspace == nullptr) return fail(CC_ERR_NULL, "workspace is NULL");
        if (!aligned(workspace, 256)) return fail(CC_ERR_ALIGN, "workspace must be 256-byte aligned");
        if (workspace_bytes < need) return fail(CC_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (cc::dense_rows_q(M, in_features, out_features)) {
        // the integers q themselves as a 16-bit codebook (exact), gathered into the operand layout and multiplied into
        // fp32 sums; scale and bias meet the finished sum
        char* wf = static_cast<char*>(workspace);
        char* book16 = wf + cc::layer_weight_frag_bytes(in_features, out_features);
        float* sums = reinterpret_cast<float*>(book16 + kIntegerBookBytes);
        CC_TRY_HIP(cc::launch_codebook_integers16(qbook, bits, K, g, dtype, book16, s), "integer codebook");
        CC_TRY_HIP(cc::launch_layer_weight_frag(book16, K, g, codes, in_features, out_features, wf, s), "integer weight");
        CC_TRY_HIP(cc::launch_layer_gemm(x, uint32_t(M), wf, dtype, in_features, out_features, scale, bias, y, sums, s),
                   "dense product");
        return CC_OK;
    }
    CC_TRY_HIP(cc::launch_layer_forward_q(x, uint32_t(M), qbook, bits, scale, K, g, codes, in_features, out_features, bias, y,
                                          dtype, static_cast<float*>(workspace), s),
               "layer forward (quantised codebook)");
    return CC_OK;
}

int cc_mfma_f16_probe(const uint16_t* A, const uint16_t* B, const float* C, float* D, uint32_t tiles, uint32_t km, void* stream)
{
    if (!A || !B || !C || !D) return fail(CC_ERR_NULL, "a required pointer is NULL");
    if (tiles == 0 || tiles > (1u << 20)) return fail(CC_ERR_SHAPE, "tiles = %u is not in 1..2^20", tiles);
    if (km != 1 && km != 2) return fail(CC_ERR_SHAPE, "km = %u is not 1 or 2", km);
    if (!aligned(A, 2) || !aligned(B, 2) || !aligned(C, 4) || !aligned(D, 4)) return fail(CC_ERR_ALIGN, "misaligned pointer");
    CC_TRY_HIP(cc::launch_mfma_f16_probe(A, B, C, D, tiles, km, static_cast<hipStream_t>(stream)), "matrix-core probe");
    return CC_OK;
}

int cc_read_stats(const void* workspace, size_t workspace_bytes, cc_stats* host_out, void* stream)
{
    if (!workspace || !host_out) return fail(CC_ERR_NULL, "a required pointer is NULL");
    if (workspace_bytes < sizeof(cc::WsHeader)) return fail(CC_ERR_WORKSPACE, "workspace too small");
    cc::WsHeader h;
    CC_TRY_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)), "stream synchronise");
    CC_TRY_HIP(hipMemcpy(&h, workspace, sizeof(h), hipMemcpyDeviceToHost), "statistics copy");
    host_out->refined_vectors = h.refined_vectors;
    host_out->skipped_vectors = h.skipped_vectors;
    host_out->assign_calls = h.assign_calls;
    host_out->scored_stages = h.window_stages;
    host_out->total_stages = h.window_total;
    host_out->fixed_point_exp = h.fixed_point_exp;
    host_out->fp16_inputs = h.x_not_f16 == 0 ? 1u : 0u;
    host_out->nonfinite_inputs = h.x_nonfinite != 0 ? 1u : 0u;
    host_out->reserved = 0;
    return CC_OK;
}

const char* cc_last_error(void) { return g_err; }

const char* cc_version(void) { return "cluscomp-gfx950 0.2"; }

}  // extern "C"
