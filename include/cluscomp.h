/*
 * cluscomp.h - C ABI of the MI355X (gfx950) clustering library.
 *
 * The library implements the clustering stage of ClusComp (Section 3.1 of the paper): Lloyd k-means
 * over the length-d sub-vectors of a weight matrix, and the codebook gather that rebuilds the matrix
 * from (codebook, codes).
 *
 * Notation: the paper's g is `d` here (sub-vector length), its n is `K` (number of centroids), its
 * k = d_in*d_out/g is `N` (number of sub-vectors), its codes q are `idx`, its codebook C is
 * `centroids`.
 *
 * Conventions shared by every call
 *   - Every pointer is a DEVICE pointer unless its comment says "host". All arrays are dense,
 *     row-major, and owned by the caller; the library never frees or keeps them.
 *   - `vectors` is the weight matrix itself: an R x C row-major fp32 matrix viewed as N = R*C/d rows of
 *     d floats (the reshape of Section 3.1; a caller who wants the paper's transposed orientation
 *     transposes before the call; cc_layer_vectors does it). Supported d: 1..16 (the paper's g runs
 *     over 4..9). The kernels are built for d = 4, 8, 16; any other length runs on zero-padded copies
 *     of the vectors and centroids kept in the workspace, which changes no distance and no mean.
 *     `vectors`, `centroids` and `out` must be 16-byte aligned, `workspace` 256-byte aligned.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default stream) and is
 *     asynchronous: results are valid once the caller has synchronised that stream. No call
 *     synchronises, allocates, or copies to the host. Concurrent calls must not share a workspace.
 *   - Arguments are validated on the host before anything is launched. A call returns CC_OK or a
 *     negative cc_status and then cc_last_error() describes the problem; nothing was enqueued in
 *     that case (except for CC_ERR_HIP, where a launch itself failed).
 *   - Same inputs give the same output bits on every run (the cluster sums are accumulated in
 *     integer fixed point, so they do not depend on scheduling order).
 *   - Every input value must be finite. The library checks: an Inf or NaN among the vectors sets
 *     cc_stats::nonfinite_inputs, such a component is left out of every cluster sum (the other components
 *     and the cluster size still count), and the code of its vector is unspecified (but below K).
 *
 * Readings of what the paper leaves open
 *   - E-step ties: the lowest centroid index wins among exactly equal distances; when two distances
 *     differ by less than the fp32 rounding of the direct form (relative 1e-6), either may win.
 *   - Empty cluster in the M-step: the centroid keeps its previous value.
 *   - Returned codes and inertia belong to the RETURNED codebook (the definition of q in
 *     Section 3.1): a fit of T iterations runs T (assign, update) pairs and one final assign.
 */
#ifndef CLUSCOMP_H
#define CLUSCOMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum cc_status {
    CC_OK = 0,
    CC_ERR_NULL = -1,      /* a required pointer is NULL */
    CC_ERR_SHAPE = -2,     /* N == 0, N >= 2^32, d not in 1..16, K == 0, K > N, K > 2^24 */
    CC_ERR_ITERS = -3,     /* iters < 0 */
    CC_ERR_ALIGN = -4,     /* a pointer violates the alignment stated above */
    CC_ERR_WORKSPACE = -5, /* workspace_bytes < cc_workspace_bytes(N, d, K) */
    CC_ERR_HIP = -6        /* the HIP runtime reported an error at launch */
} cc_status;

/*
 * Per-call options of the *_ex entry points (every other entry point behaves like its *_ex form with options =
 * NULL). Zero the struct, set struct_bytes = sizeof(cc_options), then the fields wanted. Options belong to one
 * call: nothing in the library is process-wide, so concurrent callers cannot change each other's kernels.
 *
 * assign_mode selects the E-step kernel (Section 3.1, the argmin over the centroids); every choice returns the same
 * codes, they differ in speed and exist for tests and profiling:
 *   CC_ASSIGN_AUTO        for K >= 128 the matrix cores - the fp16 MFMA with the centroids split into fp16 parts
 *                         (exact products, fp32 accumulation) when every input is an fp16 number, the fp32 MFMA
 *                         otherwise, both with a rounding guard band + direct-form refinement - and the direct form
 *                         on the vector ALUs for smaller K. For K >= 8192 (inside cc_kmeans_fit already for K >= 256
 *                         when N >= 2^19 and iters >= 5, where the ordering is paid once) vectors and centroids are
 *                         additionally visited in the order of a (norm, cosine to a fixed direction) key and a
 *                         workgroup skips the parts of the codebook that the triangle inequality rules out: a centroid
 *                         whose norm, or whose projection on the fixed direction, differs from a vector's by more than
 *                         a known upper bound of its nearest distance cannot be the nearest. The previous E-step's
 *                         codes on the same workspace - or a bootstrap pass over a guessed neighbourhood of each
 *                         vector - provide that bound; a poor bound costs time, never correctness.
 *   CC_ASSIGN_DIRECT      direct-form vector-ALU kernel only.
 *   CC_ASSIGN_MFMA_F32    fp32 MFMA kernel always, whole codebook.
 *   CC_ASSIGN_AUTO_WHOLE  as CC_ASSIGN_AUTO but always the whole codebook, and every M-step recomputed.
 *
 * profile (may be NULL): a cc_profile in which the call records the device time of its own kernels.
 */
typedef enum cc_assign_mode {
    CC_ASSIGN_AUTO = 0, CC_ASSIGN_DIRECT = 1, CC_ASSIGN_MFMA_F32 = 2, CC_ASSIGN_AUTO_WHOLE = 3
} cc_assign_mode;

typedef struct cc_profile cc_profile;   /* opaque host object */

typedef struct cc_options {
    uint32_t struct_bytes;  /* sizeof(cc_options) */
    int32_t assign_mode;    /* a cc_assign_mode */
    cc_profile *profile;    /* NULL, or see cc_profile_create */
} cc_options;

/*
 * Device time of the library's kernels, measured with HIP events recorded on the stream of the call that the
 * profile is passed to (for benchmarks: the time of the dominant kernel inside a whole fit). Each launch - or short
 * run of launches - named by a slot takes one record:
 *   CC_PROF_ESTEP_F16     the scoring kernel of the E-step on the fp16 matrix cores, one record per launch
 *   CC_PROF_ESTEP_F32     the same on the fp32 matrix cores (both are enqueued; the one whose inputs do not
 *                         qualify returns at once)
 *   CC_PROF_ESTEP_DIRECT  the direct-form E-step kernel
 *   CC_PROF_REFINE        re-decision of the guard-band vectors
 *   CC_PROF_MSTEP         all kernels of one M-step
 *   CC_PROF_ORDER         key ordering of vectors / centroids, window lists
 * cc_profile_create allocates (host memory and max_records pairs of events) and is the only profile call that does;
 * slot_mask selects the slots to record (bit s = slot s) - an event pair costs a few microseconds of stream time.
 * cc_profile_read waits for the recorded events (it synchronises with the work they bracket), adds up ms[slot]
 * (milliseconds) and launches[slot] (both host arrays of CC_PROF_SLOTS entries), reports in *dropped (host, may be
 * NULL) how many records did not fit, and empties the profile. Not for use on a stream under graph capture, and
 * one profile serves one stream at a time.
 */
typedef enum cc_profile_slot {
    CC_PROF_ESTEP_F16 = 0, CC_PROF_ESTEP_F32 = 1, CC_PROF_ESTEP_DIRECT = 2, CC_PROF_REFINE = 3, CC_PROF_MSTEP = 4,
    CC_PROF_ORDER = 5, CC_PROF_SLOTS = 6
} cc_profile_slot;
int cc_profile_create(uint32_t max_records, uint32_t slot_mask, cc_profile **out);
int cc_profile_read(cc_profile *profile, double *ms, uint32_t *launches, uint32_t *dropped);
void cc_profile_destroy(cc_profile *profile);

/* Host-only query: bytes of device workspace that cc_kmeans_fit / cc_assign / cc_lloyd_iter / cc_update
 * need for this problem size (about 12*N*d + 54*N bytes: an ordered copy of the vectors, room for two
 * copies grouped by cluster for the M-step, permutations and sort buffers, with d rounded up to 4, 8 or 16; plus one
 * more padded copy of the vectors if d is not one of those). Returns 0 for an unsupported shape. The
 * first 256 bytes keep a little state between calls (problem shape, "codes of the previous E-step are
 * present"): a workspace that held something else in between is still safe to reuse - stale state can
 * only make a call slower, not wrong. */
size_t cc_workspace_bytes(uint64_t N, uint32_t d, uint32_t K);

/*
 * Lloyd k-means (Section 3.1: the E-step / M-step iteration; Appendix B.1 runs it for 20 iterations).
 *   vectors        [N*d] in   the sub-vectors w_i
 *   init_centroids [K*d] in   centroids entering iteration 0 (e.g. a seeded subset of the vectors)
 *   centroids      [K*d] out  the codebook after `iters` updates; may alias init_centroids
 *   idx            [N]   out  q_i = argmin_k ||w_i - c_k||^2 over the RETURNED codebook
 *   inertia        [1]   out  fp64, sum_i ||w_i - c_{q_i}||^2 for the returned (codebook, codes);
 *                             may be NULL
 * iters == 0 copies init_centroids through and only assigns.
 */
int cc_kmeans_fit(const float *vectors, uint64_t N, uint32_t d, uint32_t K, int32_t iters,
                  const float *init_centroids, float *centroids, uint32_t *idx, double *inertia,
                  void *workspace, size_t workspace_bytes, void *stream);
int cc_kmeans_fit_ex(const float *vectors, uint64_t N, uint32_t d, uint32_t K, int32_t iters,
                     const float *init_centroids, float *centroids, uint32_t *idx, double *inertia,
                     void *workspace, size_t workspace_bytes, void *stream, const cc_options *options);

/*
 * E-step alone (Section 3.1): idx_i = argmin_k ||w_i - c_k||^2, and optionally the objective
 * sum_i ||w_i - c_{idx_i}||^2 (fp64, device, may be NULL).
 */
int cc_assign(const float *vectors, uint64_t N, uint32_t d, const float *centroids, uint32_t K,
              uint32_t *idx, double *inertia, void *workspace, size_t workspace_bytes, void *stream);
int cc_assign_ex(const float *vectors, uint64_t N, uint32_t d, const float *centroids, uint32_t K,
                 uint32_t *idx, double *inertia, void *workspace, size_t workspace_bytes, void *stream,
                 const cc_options *options);

/*
 * One Lloyd iteration (Section 3.1: an E-step followed by an M-step), the unit the fit repeats:
 *   idx_i      = argmin_k ||w_i - c_k||^2 over the centroids as passed in,
 *   centroids <- per-cluster means of those assignments, in place (empty clusters keep their value),
 *   inertia    (fp64, device, may be NULL) = sum_i ||w_i - c_{idx_i}||^2 against the centroids as passed in,
 *   counts [K] (uint32, may be NULL) = cluster sizes.
 * The result is bit-identical to cc_assign followed by cc_update; it is faster because the cluster
 * sums are accumulated by the assignment kernel while the vectors are on chip.
 */
int cc_lloyd_iter(const float *vectors, uint64_t N, uint32_t d, float *centroids, uint32_t K, uint32_t *idx,
                  double *inertia, uint32_t *counts, void *workspace, size_t workspace_bytes, void *stream);
int cc_lloyd_iter_ex(const float *vectors, uint64_t N, uint32_t d, float *centroids, uint32_t K, uint32_t *idx,
                     double *inertia, uint32_t *counts, void *workspace, size_t workspace_bytes, void *stream,
                     const cc_options *options);

/*
 * M-step alone (Section 3.1): centroids_k = mean of the vectors with idx_i == k; a cluster without
 * members keeps prev_centroids_k. Every idx_i must be < K (checked on the device: offending vectors
 * are skipped and counted in the workspace statistics). `centroids` may alias `prev_centroids`.
 * `counts` [K] (out, uint32, may be NULL) receives the cluster sizes.
 */
int cc_update(const float *vectors, uint64_t N, uint32_t d, const uint32_t *idx,
              const float *prev_centroids, uint32_t K, float *centroids, uint32_t *counts,
              void *workspace, size_t workspace_bytes, void *stream);
int cc_update_ex(const float *vectors, uint64_t N, uint32_t d, const uint32_t *idx,
                 const float *prev_centroids, uint32_t K, float *centroids, uint32_t *counts,
                 void *workspace, size_t workspace_bytes, void *stream, const cc_options *options);

/*
 * Reconstruction (Section 3.1; the gather `codebook[code]` of the paper's layer listing):
 * out_i = centroids_{idx_i}, i.e. the R x C matrix again when `out` is viewed row-major.
 * Pure data movement, bit-exact. An idx_i >= K is clamped to K-1 (never read out of bounds).
 */
int cc_decode(const float *centroids, uint32_t K, uint32_t d, const uint32_t *idx, uint64_t N,
              float *out, void *stream);

/*
 * Counters that the last cc_kmeans_fit / cc_assign / cc_update on `workspace` left behind.
 * Copies them to `host_out` (host pointer) with a synchronous device-to-host copy after
 * synchronising `stream`; meant for tests and logging, not for the hot path.
 */
typedef struct cc_stats {
    uint64_t refined_vectors;  /* vectors whose fast-path decision was inside the guard band and was
                                  re-decided with direct-form distances (summed over all assigns) */
    uint64_t skipped_vectors;  /* vectors with idx >= K seen by an update */
    uint64_t assign_calls;     /* assign passes run */
    uint64_t scored_stages;    /* window pruning: codebook tiles (32 centroids) scored, summed over the
                                  512-vector tiles of all assigns; 0 when pruning did not run */
    uint64_t total_stages;     /* the same sum if every tile had scored the whole codebook */
    int32_t  fixed_point_exp;  /* e: cluster sums are held as round(x * 2^e) in int64 */
    uint32_t fp16_inputs;      /* 1 if the vectors of the last call qualified for the fp16 matrix-core kernels
                                  (|x| < 2^15 and every |x| >= 2^-14 an fp16 number), else 0 */
    uint32_t nonfinite_inputs; /* 1 if some input of the last call was Inf or NaN (a violated precondition) */
    uint32_t reserved;
} cc_stats;
int cc_read_stats(const void *workspace, size_t workspace_bytes, cc_stats *host_out, void *stream);

/* ------------------------------------------------------------------------------------------------
 * The compressed linear layer (Section 3.1 footnote, Section 3.2, and the paper's layer listing).
 *
 * A linear layer's weight is stored [out_features, in_features] by the framework. What is clustered is
 * its transpose, W[in_features, out_features] row-major, each row zero-padded by
 * deficiency = (g - out_features % g) % g columns and cut into vectors of length g; the layer keeps a
 * codebook [K, g] in a 16-bit float format and num_codes = in_features * (out_features + deficiency) / g
 * unsigned 16-bit codes (hence K <= 65536), and rebuilds W by gathering codebook rows and cutting the
 * padding columns off again. Element types are given as a cc_dtype.
 */
typedef enum cc_dtype { CC_F32 = 0, CC_F16 = 1, CC_BF16 = 2 } cc_dtype;

/* Host-only arithmetic of the layer's constructor. */
uint32_t cc_layer_deficiency(uint32_t out_features, uint32_t g);
uint64_t cc_layer_num_codes(uint64_t in_features, uint64_t out_features, uint32_t g);

/*
 * The vectors to cluster (Section 3.1 footnote): weight [out_features * in_features] (weight_dtype) is
 * transposed, every row of the transpose is zero-padded to out_features + deficiency columns, and the
 * result is written as fp32: vectors [num_codes * g], ready for cc_kmeans_fit with N = num_codes, d = g.
 */
int cc_layer_vectors(const void *weight, int weight_dtype, uint32_t out_features, uint32_t in_features,
                     uint32_t g, float *vectors, void *stream);

/*
 * Storage formats (Section 3.2): centroids [K * g] fp32 -> codebook [K * g] in codebook_dtype (CC_F16 or
 * CC_BF16, round to nearest even); idx [num_codes] uint32 -> codes [num_codes] uint16. K <= 65536; an idx
 * value >= K is clamped to K - 1. Either half may be skipped by passing NULL for both of its pointers.
 */
int cc_layer_pack(const float *centroids, uint32_t K, uint32_t g, void *codebook, int codebook_dtype,
                  const uint32_t *idx, uint64_t num_codes, uint16_t *codes, void *stream);

/*
 * Reconstruction (layer listing, forward: gather, view as in_features rows, cut the padding):
 * weight [in_features * out_features] in the codebook's dtype, weight[r][c] = codebook[codes[(r * width + c) / g]]
 * [(r * width + c) % g] with width = out_features + deficiency. Pure data movement, bit-exact.
 * A code >= K is clamped to K - 1. `dtype` may be CC_F32, CC_F16 or CC_BF16.
 */
int cc_layer_weight(const void *codebook, int dtype, uint32_t K, uint32_t g, const uint16_t *codes,
                    uint32_t in_features, uint32_t out_features, void *weight, void *stream);

/*
 * Forward pass of the layer (layer listing): y [M * out_features] = x [M * in_features] . W (+ bias), with W
 * as rebuilt by cc_layer_weight. x, codebook, bias (may be NULL) and y share one 16-bit dtype (CC_F16 or
 * CC_BF16); products are exact, accumulation is fp32, y is rounded once (to nearest even). in_features must be
 * a multiple of 8, M <= 2^22; x, y and codebook 16-byte aligned. Two routes, chosen by the shape alone (the
 * second from M = 128 on, for layers of 2^24 weights or more already from M = 65, and from M = 33 for layers of
 * 2^25 weights or more with out_features >= 2 * in_features):
 *   few rows (decoding): W is never written to memory: codebook rows are gathered straight into matrix-core
 *     operand tiles (up to 4 rows with g = 4: one lane per code column and plain multiply-adds instead). The
 *     summation order is fixed: same inputs, same bits. Workspace: fp32 partial sums of the in-feature slices
 *     that fill the chip when M is small.
 *   many rows (prefill, wide decoding batches): the listing's own order. W is rebuilt once into the workspace
 *     (in the register layout of the matrix cores' operand, padded to whole operands) and multiplied by the
 *     library's own matrix-core kernel: 256 x 256 tiles of y, fp32 accumulation in a fixed order, bias added to the
 *     finished sum, one rounding. Tiles that do not fill a round of the chip are also split along the contraction
 *     and their fp32 partial tiles added in a fixed order by a second kernel. Workspace: W plus those partial tiles.
 * cc_layer_forward_workspace_bytes(M, in_features, out_features) bytes, 256-byte aligned; may be NULL if that is 0.
 */
size_t cc_layer_forward_workspace_bytes(uint64_t M, uint32_t in_features, uint32_t out_features);
int cc_layer_forward(const void *x, uint64_t M, const void *codebook, int dtype, uint32_t K, uint32_t g,
                     const uint16_t *codes, uint32_t in_features, uint32_t out_features, const void *bias,
                     void *y, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Gradient of the codebook (the only trainable tensor of the layer, Sections 3.2-3.3): every weight entry
 * is a copy of one codebook entry, so grad_codebook [K * g] (fp32) [k][j] is the sum of grad_weight
 * [in_features * out_features] (grad_dtype) over the entries rebuilt from codebook[k][j]. Sums are
 * accumulated in 64-bit fixed point scaled from max |grad|: deterministic, exact for 16-bit gradients, and
 * within 2^-38 * max |grad| per term otherwise. Gradients must be finite.
 * A 16-bit gradient of a layer with at least 2^20 codes, g = 4, 8 or 16 and out_features a multiple of g is read
 * where it lies if grad_weight is 16-byte and codes 4-byte aligned (same bits, about a third of the time);
 * every other case goes through an fp32 copy of the gradient in the workspace.
 * Workspace: cc_workspace_bytes(num_codes, g, K) bytes.
 */
int cc_layer_codebook_grad(const void *grad_weight, int grad_dtype, uint32_t in_features, uint32_t out_features,
                           const uint16_t *codes, uint32_t K, uint32_t g, float *grad_codebook,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same gradient for training loops (Section 3.3: only the codebook is trained, the codes of a layer never
 * change): cc_layer_grad_plan orders the code positions by cluster once; cc_layer_codebook_grad_planned then
 * reads every gradient entry once, straight from grad_weight, and adds each cluster's entries in fp64 in a
 * fixed order (same inputs, same bits; each sum is within count * 2^-53 * sum |terms| of exact before its one
 * rounding to fp32, i.e. the rounded exact sum for 16-bit gradients in practice). Codes >= K are left out.
 *   plan       device memory, cc_layer_grad_plan_bytes(num_codes, K) bytes, 256-byte aligned; written by
 *              cc_layer_grad_plan, read-only afterwards, owned by the caller for as long as the codes live.
 *   workspace  scratch: cc_layer_grad_plan_workspace_bytes(num_codes) for the build,
 *              cc_layer_codebook_grad_planned_workspace_bytes(num_codes, K, g) for each gradient; 256-byte aligned.
 * grad_weight must be 16-byte aligned; K <= 65536, num_codes < 2^32. A plan built for another (num_codes, K) is
 * detected on the device: grad_codebook then comes back as NaN.
 */
size_t cc_layer_grad_plan_bytes(uint64_t num_codes, uint32_t K);
size_t cc_layer_grad_plan_workspace_bytes(uint64_t num_codes);
int cc_layer_grad_plan(const uint16_t *codes, uint64_t num_codes, uint32_t K, void *plan, size_t plan_bytes,
                       void *workspace, size_t workspace_bytes, void *stream);
size_t cc_layer_codebook_grad_planned_workspace_bytes(uint64_t num_codes, uint32_t K, uint32_t g);
int cc_layer_codebook_grad_planned(const void *grad_weight, int grad_dtype, uint32_t in_features,
                                   uint32_t out_features, uint32_t K, uint32_t g, const void *plan, size_t plan_bytes,
                                   float *grad_codebook, void *workspace, size_t workspace_bytes, void *stream);

/*
 * One layer in one call (Sections 3.1-3.2): cc_layer_vectors, then the centroids start from the vectors listed in
 * init_ids [K] (indices < num_codes, e.g. a seeded sample without replacement drawn by the caller; an index past
 * the end is clamped), `iters` Lloyd iterations (cc_kmeans_fit), then cc_layer_pack: codebook [K * g] in
 * codebook_dtype and codes [num_codes] uint16 for the layer listing; inertia (fp64, device) may be NULL.
 * Bit-identical to calling those entry points one after the other. K <= min(65536, num_codes).
 * Workspace: cc_layer_compress_workspace_bytes(...) bytes (the fp32 vectors, centroids and codes of the
 * intermediate steps plus the clustering workspace); 0 for an unsupported shape.
 */
size_t cc_layer_compress_workspace_bytes(uint32_t out_features, uint32_t in_features, uint32_t g, uint32_t K);
int cc_layer_compress(const void *weight, int weight_dtype, uint32_t out_features, uint32_t in_features, uint32_t g,
                      uint32_t K, int32_t iters, const uint32_t *init_ids, void *codebook, int codebook_dtype,
                      uint16_t *codes, double *inertia, void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------------------------------
 * Uniformly quantised codebook (the paper's inference-only variant: "#Bits for Codebook" 8 and 4 in its
 * throughput and perplexity tables; the grid is the symmetric uniform one of Section 2, with one deviation:
 * Section 2 prints 2^bits - 1 under the scale, which together with its own clamp to [-2^(bits-1), 2^(bits-1) - 1]
 * would clip every entry above half the range, so the scale here divides by 2^(bits-1) - 1 and the clamp is a
 * safeguard only).
 * One scale per codebook: s = max|c| / (2^(bits-1) - 1), q = clamp(round_to_nearest_even(c / s),
 * -2^(bits-1), 2^(bits-1) - 1), both in fp32; the dequantised entry is q * s (fp32) rounded to the layer's
 * 16-bit format. Storage: bits = 8: int8 [K * g]; bits = 4: two's-complement nibbles, element e in byte
 * e / 2, low nibble first, ceil(K * g / 2) bytes. A codebook of at most 128 KB (K = 65536, g = 4 at 4 bits)
 * is held in LDS by persistent workgroups, which lifts the one-cache-miss-per-code limit of the 16-bit path.
 */

/* centroids [K * g] fp32 -> qbook (layout above) and scale [1] (device, fp32). `scratch` is 4 bytes of
 * device memory (4-byte aligned) used for the maximum. bits must be 8 or 4. */
int cc_codebook_quantize(const float *centroids, uint32_t K, uint32_t g, int bits, void *qbook, float *scale,
                         void *scratch, void *stream);

/* cc_layer_weight with the quantised codebook: weight [in_features * out_features] in `dtype` (CC_F16 or
 * CC_BF16), bit-exact with respect to the dequantisation rule above. */
int cc_layer_weight_q(const void *qbook, int bits, const float *scale, uint32_t K, uint32_t g,
                      const uint16_t *codes, uint32_t in_features, uint32_t out_features, int dtype, void *weight,
                      void *stream);

/* cc_layer_forward with the quantised codebook (x, bias, y in `dtype`): y = s * (x . Q) (+ bias), where Q is the
 * weight rebuilt from the integers q themselves. The products x * q are exact, the sum is fp32, the scale
 * multiplies the finished sum, and y is rounded once - so this is slightly more accurate than a product with
 * the 16-bit weight of cc_layer_weight_q, whose entries are each rounded to 16 bits. Same contract otherwise,
 * both routes included (the second from M = 65 on, from M = 33 on for layers of 2^24 weights or more, from M = 16
 * on for layers of 2^25 weights or more with out_features >= 2 * in_features): there the integers q become a 16-bit
 * codebook (exact), the weight is rebuilt from it into the matrix cores' operand layout, and the same matrix-core
 * kernel applies scale and bias to the finished fp32 sum and rounds once.
 * Workspace: cc_layer_forward_q_workspace_bytes(M, in_features, out_features). */
size_t cc_layer_forward_q_workspace_bytes(uint64_t M, uint32_t in_features, uint32_t out_features);
int cc_layer_forward_q(const void *x, uint64_t M, const void *qbook, int bits, const float *scale, uint32_t K,
                       uint32_t g, const uint16_t *codes, uint32_t in_features, uint32_t out_features,
                       const void *bias, void *y, int dtype, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Diagnostic, for tests: what the fp16 matrix core (v_mfma_f32_32x32x16_f16) returns for caller-chosen operands,
 * chained as the default E-step of Section 3.1's argmin chains it (km = 1 or 2 instructions, the accumulator preset
 * per output row). The E-step's guard band assumes that this result is within 8 * 2^-24 * S of the exact sum, S
 * being the sum over the nonzero products a * b of max(|a|, 2^-14) * max(|b|, 2^-14) plus |c|; the hardware manuals
 * do not state the accumulation order, so a GPU test pins the bound with this call against exact arithmetic.
 *   A [tiles * 32 * 16 * km], B [tiles * 32 * 16 * km]  fp16 bit patterns: row m of A against row n of B
 *   C [tiles * 32]  fp32, start value of the accumulator for output row m
 *   D [tiles * 32 * 32]  out, fp32: D[m][n] = C[m] + sum_q A[m][q] * B[n][q] as the instruction computes it
 */
int cc_mfma_f16_probe(const uint16_t *A, const uint16_t *B, const float *C, float *D, uint32_t tiles, uint32_t km,
                      void *stream);

/* Thread-local description of the last error returned on this thread (host pointer, static storage). */
const char *cc_last_error(void);

/* Library version string (host pointer, static storage). */
const char *cc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CLUSCOMP_H */
