/*
 * libdgc -- the per-worker hot path of Deep Gradient Compression
 * (arXiv 1712.01887) as HIP kernels for gfx950 behind a C ABI.
 *
 * One call of dgc_compress is one iteration of Algorithm 3 (Appendix D) on one
 * worker, from the clipping line to the mask lines, for a whole gradient set
 * stored flat; dgc_decompress_accumulate is the sum in its all-reduce line.
 *
 * Conventions
 *   - Every function returns a dgc_status (0 = success, negative = error).
 *     No exception or abort crosses this boundary.
 *   - "device" pointers address GPU memory of the current HIP device, "host"
 *     pointers address ordinary process memory.  The library never takes
 *     ownership of a buffer and never frees one.
 *   - All device work is enqueued on the caller's stream (a hipStream_t passed
 *     as void*, NULL = the default stream) and is asynchronous; only
 *     dgc_get_diagnostics waits for the stream.
 *   - Flat layout: tensor j of the set occupies elements
 *     [offsets[j], offsets[j+1]) of g, u, v and of the dense aggregate.
 *     Element type is IEEE binary32; indices are int32 (n < 2^31).
 *   - Arithmetic is binary32 with one rounding per operation (no fused
 *     multiply-add, denormals kept); the clipping norm is accumulated in
 *     binary64.
 */
#ifndef DGC_H_
#define DGC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t dgc_status;
enum {
  DGC_OK = 0,
  DGC_ERR_INVALID_ARG = -1, /* null pointer, value out of range                */
  DGC_ERR_ALIGNMENT = -2,   /* g, u, v or dense not 16-byte aligned            */
  DGC_ERR_CAPACITY = -3,    /* workspace too small, too many payloads/tensors  */
  DGC_ERR_HIP = -4,         /* a HIP runtime call failed                       */
  DGC_ERR_STATE = -5        /* call order violated                             */
};

/* dgc_config.flags */
enum {
  DGC_FLAG_NESTEROV = 1u << 0,          /* Algorithm 4: U <- m(U+G); V <- V+U+G          */
  DGC_FLAG_NO_FACTOR_MASKING = 1u << 1, /* leave U untouched (Section 3.3 switched off)   */
  DGC_FLAG_EXACT_SELECT = 1u << 2,      /* threshold from the whole tensor, not a sample  */
  DGC_FLAG_DETERMINISTIC_ACCUMULATE = 1u << 3, /* receive side adds workers in order      */
  DGC_FLAG_SORTED_OUTPUT = 1u << 4      /* pairs of a tensor in ascending index order; the
                                           payload is then identical on every run, and a full
                                           region keeps the lowest indices                      */
};

/* dgc_diagnostics.flags */
enum {
  DGC_DIAG_OVERFLOW = 1u << 0,   /* some tensor had more passes than payload capacity */
  DGC_DIAG_NONFINITE = 1u << 1,  /* the clipping norm was not finite                  */
  DGC_DIAG_BAD_INDEX = 1u << 2,  /* a payload index fell outside [0, n): skipped      */
  DGC_DIAG_UNSORTED = 1u << 3    /* dgc_encode met a region that is not ascending     */
};

/*
 * Arguments of the method (Algorithm 3 "Require": momentum m, node count N;
 * Appendix C: global clipping threshold; Section 4.1: density = 1 - sparsity;
 * Section 5: the threshold is estimated on a sample of 0.1 % .. 1 %).
 */
typedef struct dgc_config {
  float momentum;        /* m                                                        */
  float clip_threshold;  /* thr_G; the local one is thr_G / sqrt(N); <= 0: no clip   */
  int32_t num_workers;   /* N >= 1                                                   */
  uint32_t flags;        /* DGC_FLAG_*                                               */
  double density;        /* d in (0, 1]; k_j = clamp(ceil(d * n_j), 1, n_j)          */
  double sample_ratio;   /* wanted sample size as a fraction of n_j (0.01)           */
  int32_t sample_min;    /* lower clamp of the sample size (4096)                    */
  int32_t sample_max;    /* upper clamp of the sample size (32768)                   */
  int32_t sample_block;  /* consecutive elements per draw, power of two <= 64 (32)   */
  float scale_override;  /* test hook: NaN = unused, else replaces the clip scale    */
  uint64_t seed;         /* seed of the counter-based sample positions               */
  float refine_alpha;    /* Section 5 re-threshold: when more than alpha * k_j elements of a
                            tensor pass the sampled threshold, the threshold is recomputed
                            exactly from those that passed; 0 = off, otherwise >= 1 (2)  */
  uint32_t reserved;     /* zero                                                     */
} dgc_config;

typedef struct dgc_diagnostics {
  double norm;     /* L2 norm of g over the whole set (NaN when clipping is off) */
  float scale;     /* factor applied to g                                         */
  uint32_t flags;  /* DGC_DIAG_*                                                  */
} dgc_diagnostics;

typedef struct dgc_handle dgc_handle;

/* Fill *cfg with m = 0.9, no clipping, N = 1, d = 0.001, sampling 1 % clamped to
 * [4096, 32768] in blocks of 32, seed 0, no re-threshold. */
dgc_status dgc_config_default(dgc_config* cfg);

/* Text for a status code (static storage). */
const char* dgc_status_string(dgc_status s);
/* Detail of the most recent DGC_ERR_HIP on the calling thread: which step failed and
 * the runtime's message.  Thread-local storage, valid until the next failure. */
const char* dgc_last_error_string(void);

/*
 * Create the host-side description of a gradient set.
 *   offsets_host: host, num_tensors + 1 ascending element offsets, offsets[0] = 0,
 *                 every tensor non-empty, offsets[num_tensors] = n < 2^31.
 * Allocates host memory only.  The handle is not thread-safe.
 */
dgc_status dgc_create(dgc_handle** out, const dgc_config* cfg, int32_t num_tensors,
                      const int64_t* offsets_host);
dgc_status dgc_destroy(dgc_handle* h);

/*
 * Workspaces.  The device workspace passed to dgc_compress and to the region calls of the
 * receive side holds tables that the library uploads (tile and work lists, the selection plan
 * of the current density, the payload layout) the first time a handle meets it, and again
 * when the density or the layout changes.  The handle remembers on the host what it has
 * uploaded where, so:
 *   - give every handle a workspace of its own on the hot path.  A workspace may pass from one
 *     handle to another between calls (never between calls that overlap in time): the library
 *     notices and uploads the new owner's tables again, which costs several host-to-device
 *     copies per change of owner;
 *   - a workspace that was freed, overwritten by the caller, or allocated again at the same
 *     address must be announced with dgc_invalidate_workspace before its next use: the
 *     library cannot see that its tables are gone;
 *   - uploads cannot be captured into a HIP graph.  A call that would have to upload while
 *     its stream is being captured returns DGC_ERR_STATE and enqueues nothing: make the first
 *     call on a workspace, and the first one after dgc_set_density or a change of payload
 *     layout, outside the capture.
 * dgc_invalidate_workspace forgets everything the handle believes about its workspace; the
 * next call uploads all tables again.  Host only.
 */
dgc_status dgc_invalidate_workspace(dgc_handle* h);

/*
 * Density control (Section 3.3 "warm-up training"; Section 4.1 lists the
 * sparsities 75 %, 93.75 %, 98.4375 %, 99.6 %, 99.9 %).  Host only: recomputes
 * k_j and the sample plan; the next dgc_compress uploads the new plan.
 */
dgc_status dgc_set_density(dgc_handle* h, double density);
/* Replace the warm-up table (host, len >= 1 densities in (0, 1]).  The default
 * table is {0.25, 0.0625, 0.015625, 0.004, 0.001}. */
dgc_status dgc_set_warmup_schedule(dgc_handle* h, const double* densities_host, int32_t len);
/* Iterations every table entry is held (default 1).  The paper's runs hold a warm-up
 * sparsity for one epoch (Section 4.1: a warm-up period of 4 epochs for the four values
 * before the final one): pass the iterations of an epoch. */
dgc_status dgc_set_warmup_stage_length(dgc_handle* h, int64_t iterations_per_stage);
/* density <- table[min(iteration / stage length, len - 1)]. */
dgc_status dgc_set_iteration_density(dgc_handle* h, int64_t iteration);

/*
 * Test hook for the clipping scale of Appendix C (equation 12): a finite value replaces the
 * factor min(1, thr_local / ||g||) in the following dgc_compress calls (the norm is still
 * computed and reported when clipping is on), NaN returns to the computed one.  Same meaning
 * as dgc_config.scale_override.  Host only.  Errors: INVALID_ARG (null handle, infinity).
 */
dgc_status dgc_set_scale_override(dgc_handle* h, float scale);

/*
 * Host arithmetic of tensor j under the current density (any pointer may be NULL):
 *   k            = clamp(ceil(d * n_j), 1, n_j)
 *   sample_count = candidates the threshold is selected from (n_j when the whole
 *                  tensor is used, else draws * sample_block)
 *   rank         = 0-based descending rank whose magnitude becomes the threshold
 *   draws        = number of sampled blocks (0 when the whole tensor is used)
 */
dgc_status dgc_query_plan(const dgc_handle* h, int32_t j, int64_t* k, int64_t* sample_count,
                          int64_t* rank, int64_t* draws);

/* Bytes of device workspace dgc_compress needs for this set (any density). */
dgc_status dgc_workspace_bytes(const dgc_handle* h, size_t* bytes);

/*
 * Bytes of a workspace that also holds two staging arrays of n floats each (Section 4,
 * warm-up training: 25 % down to 0.4 % of the elements are sent during the first epochs).
 * Given a workspace of at least this size, dgc_compress at a density above 0.5 % masks u
 * and v inside its streaming pass and parks the selected values in the staging arrays, so
 * that the emit pass does not come back to u and v (1017 -> about 600 us at 25 % on a
 * 122 M-element set); every region of the payload is then in ascending index order.  With
 * the smaller workspace, or with refine_alpha > 0, the same results are computed the slower
 * way.  Results do not depend on which workspace is given.
 */
dgc_status dgc_workspace_bytes_warmup(const dgc_handle* h, size_t* bytes);

/*
 * A payload layout for `density`: out_offsets_host (host, num_tensors + 1) receives
 * the start of each tensor's pair region, capacity_j = min(n_j, max(8 k_j, k_j + 256)).
 */
dgc_status dgc_recommended_payload_layout(const dgc_handle* h, double density,
                                          int64_t* out_offsets_host);

/*
 * One iteration on one worker (Algorithm 3, or Algorithm 4 with DGC_FLAG_NESTEROV):
 *   scale  = clip ? min(1, (thr_G / sqrt N) / ||g||_2) : 1          (Appendix C)
 *   u'     = m u + scale g ;  v' = v + u'                            (equation 7)
 *   thr_j  = magnitude of descending rank r_j among the sampled |v'| of tensor j,
 *            or of the whole tensor when it is small or EXACT_SELECT (Section 5)
 *   if refine_alpha > 0 and more than refine_alpha * k_j elements pass: thr_j =
 *            magnitude of descending rank k_j among those that passed    (Section 5)
 *   keep   = |v'| > thr_j  (strict)                                  (Algorithm 3)
 *   emit (global flat index, v') for kept elements; v <- keep ? 0 : v';
 *   u <- keep ? 0 : u'                                               (Section 3.3)
 *
 *   g          device, n floats, read only (clipping is folded into `scale`)
 *   u, v       device, n floats, updated in place; zero them before iteration 0
 *   out_idx    device, int32[out_offsets_host[num_tensors]]
 *   out_val    device, float[same]
 *   out_offsets_host  host, num_tensors + 1 ascending starts of each tensor's pair
 *              region; read during the call (the caller may reuse it afterwards)
 *   out_counts device, int32[num_tensors]: elements of tensor j that passed the
 *              mask.  Pairs [out_offsets[j], out_offsets[j] + min(count_j, capacity_j))
 *              are valid: the same pairs in the same order on every run, the parts of
 *              consecutive blocks of 32768 elements in index order, ascending throughout
 *              with DGC_FLAG_SORTED_OUTPUT (and, as it happens, whenever the staging arrays of
 *              dgc_workspace_bytes_warmup are in use, and up to a density of 0.5 % without the
 *              re-threshold: only the flag is a promise).  An element that passed but found
 *              the region full is neither emitted nor cleared (it stays in u, v) and
 *              DGC_DIAG_OVERFLOW is raised; in an ascending region those are the highest
 *              indices.
 *   out_thr    device, float[num_tensors], or NULL
 *   iteration  t: with the seed and the tensor index it fixes the sample positions
 *   workspace  device, >= dgc_workspace_bytes (or dgc_workspace_bytes_warmup), 256-byte
 *              aligned; it must not be shared by calls that may overlap in time (see
 *              "Workspaces" above)
 * Errors: INVALID_ARG (null, bad layout), ALIGNMENT, CAPACITY (workspace), HIP, STATE (tables
 * would have to be uploaded while the stream is being captured).
 */
dgc_status dgc_compress(dgc_handle* h, const float* g, float* u, float* v, int32_t* out_idx,
                        float* out_val, const int64_t* out_offsets_host, int32_t* out_counts,
                        float* out_thr, uint64_t iteration, void* workspace,
                        size_t workspace_bytes, void* stream);

/*
 * For callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  dgc_compress with the workspace argument replaced
 * by an array of 8 MiB that is part of the library (static device memory: every GPU the
 * process uses holds its own copy until the process ends), which serves gradient sets of up
 * to about 30 M elements (the ResNet-50-shaped set needs 6 MiB).  Same arguments, results and
 * errors as dgc_compress otherwise, and
 *   CAPACITY   dgc_workspace_bytes of the handle exceeds the array (dgc_last_error_string says
 *              by how much): use dgc_compress with a workspace of the caller's;
 *   HIP        the array's address could not be obtained.
 * The call allocates nothing and frees nothing: it asks the runtime for the array's address the
 * first time it runs on a device and launches the kernels of dgc_compress.  Like dgc_compress, it
 * uploads the handle's tables (asynchronous host-to-device copies) on the handle's first call, after
 * dgc_set_density or a change of payload layout, and whenever another handle has used the array
 * in between -- calls that are refused (STATE) while the stream is being captured; every other
 * call only launches kernels.  All calls on one GPU share that GPU's array, whatever their handle or
 * stream: calls that may overlap in time on one GPU race, and the caller must order them.  The
 * array keeps the last call's contents; what has to start at zero is cleared by the library.
 * dgc_get_diagnostics with workspace = NULL reads the record of the last such call on the current
 * device.
 */
dgc_status dgc_compress_static(dgc_handle* h, const float* g, float* u, float* v, int32_t* out_idx,
                               float* out_val, const int64_t* out_offsets_host, int32_t* out_counts,
                               float* out_thr, uint64_t iteration, void* stream);

/* Copy norm, scale and flags of the last dgc_compress that used `workspace` to the
 * host (workspace = NULL: of the last dgc_compress_static on the current device).  Waits for
 * `stream`. */
dgc_status dgc_get_diagnostics(dgc_handle* h, const void* workspace, dgc_diagnostics* out_host,
                               void* stream);

/*
 * Receive side (the sum of Algorithm 3's all-reduce line; no division by N, the
 * 1/(N b) factor is already inside every worker's gradient):
 *   for each payload w, each pair p < pair_counts_host[w]:
 *       dense[idx_w[p]] += val_w[p]
 *   dense        device, n floats, accumulated into (zero it for a fresh sum)
 *   num_payloads 1 .. 64
 *   idx_ptrs_host, val_ptrs_host   host arrays of num_payloads device pointers
 *   pair_counts_host               host, pairs in each payload (>= 0)
 * Pairs with an index outside [0, n) are skipped and flagged in *diag_flags_dev
 * (device uint32, may be NULL).  Without DGC_FLAG_DETERMINISTIC_ACCUMULATE the
 * additions are hardware float atomics in arbitrary order; with it, workers are
 * added in the order given and every index of one payload must be distinct.
 */
dgc_status dgc_decompress_accumulate(dgc_handle* h, float* dense, int64_t n, int32_t num_payloads,
                                     const int32_t* const* idx_ptrs_host,
                                     const float* const* val_ptrs_host,
                                     const int64_t* pair_counts_host, uint32_t* diag_flags_dev,
                                     void* stream);

/*
 * The same sum taken straight from dgc_compress outputs, with no host round trip:
 * payload w is (idx_w, val_w, counts_w) in the per-tensor region layout
 * `out_offsets_host`; counts_w is the device int32[num_tensors] written by
 * dgc_compress (clamped to each region's capacity here).
 *   workspace    device workspace of this handle (holds the layout copy)
 * The regions must be as dgc_compress of this library writes them (the parts of
 * consecutive blocks of 32768 elements of a tensor follow each other in index order; the
 * order inside a part is free, the indices of one payload are distinct).  The payloads are
 * merged by element range in on-chip memory, workers added in the order given, without
 * float atomics, which gives the result of the plain definition bit for bit at every
 * density: up to 0.5 %, as long as the payloads together let expect no more than 6144 pairs
 * in 131072 elements (density x payloads x 131072 x 1.25), a workgroup touches only the
 * elements that occur in a range of up to 131072; otherwise (the warm-up densities of
 * Section 4, or many payloads) it keeps one part's whole range of
 * `dense` on chip, after a launch that finds every payload's pairs of every part.  A
 * region laid out otherwise gives wrong sums (never an access out of bounds); for
 * arbitrary pair lists there is dgc_decompress_accumulate.
 */
dgc_status dgc_decompress_accumulate_regions(dgc_handle* h, float* dense, int32_t num_payloads,
                                             const int32_t* const* idx_ptrs_host,
                                             const float* const* val_ptrs_host,
                                             const int32_t* const* count_ptrs_host,
                                             const int64_t* out_offsets_host, void* workspace,
                                             size_t workspace_bytes, void* stream);

/*
 * The aggregate of an iteration written in place of the one before (Algorithm 3, the
 * all-reduce line: G_t is a fresh sum of the N sparse gradients every iteration):
 *       dense <- sum over the given payloads, zero wherever none of them has an index,
 * provided that `dense` is zero outside the indices of the `previous` payloads (typically
 * those of the previous call, whose index and count arrays must still be intact;
 * num_previous = 0: `dense` is zero everywhere, as before the first iteration).  One launch
 * does what dgc_dense_clear_regions followed by dgc_decompress_accumulate_regions does: where
 * a workgroup touches only the elements that occur (see above) the sums start from zero instead
 * of the scattered contents of `dense`, and indices of the previous payloads that do not recur
 * are set to zero; otherwise (and in the call that follows such a call, whose previous payloads
 * are long), the whole of `dense` is written once and read never, and `previous` is ignored.
 * Workers are added in the order given; the result is bit for bit that of clearing and
 * accumulating.  Arguments and the regions' layout as for dgc_decompress_accumulate_regions;
 * the previous payloads have the same layout.
 */
dgc_status dgc_decompress_replace_regions(dgc_handle* h, float* dense, int32_t num_payloads,
                                          const int32_t* const* idx_ptrs_host,
                                          const float* const* val_ptrs_host,
                                          const int32_t* const* count_ptrs_host, int32_t num_previous,
                                          const int32_t* const* previous_idx_ptrs_host,
                                          const int32_t* const* previous_count_ptrs_host,
                                          const int64_t* out_offsets_host, void* workspace,
                                          size_t workspace_bytes, void* stream);

/*
 * dense[idx] = 0 for every pair of the given region-layout payloads: returns a
 * dense aggregate to all-zero after it has been consumed at the cost of the
 * payload size instead of a full fill.  Arguments as above.  Above a density of 0.5 % (or with
 * many payloads, see above) the regions must be as dgc_compress writes them: the indices of a part are
 * marked in a bitmap on chip and every 64-byte sector with a marked element is written
 * once, whole (its other elements are read and written back unchanged).
 */
dgc_status dgc_dense_clear_regions(dgc_handle* h, float* dense, int32_t num_payloads,
                                   const int32_t* const* idx_ptrs_host,
                                   const int32_t* const* count_ptrs_host,
                                   const int64_t* out_offsets_host, void* workspace,
                                   size_t workspace_bytes, void* stream);

/*
 * Receive side fused with the optimizer step (the last line of Algorithm 3 with plain SGD,
 * theta <- theta - lr * G_t, G_t being the sum of the N sparse gradients): for every pair
 *       theta[idx] -= lr * val
 * so that no dense aggregate is formed and none has to be cleared.  Arguments as for
 * dgc_decompress_accumulate / dgc_decompress_accumulate_regions, theta (device, n floats) in
 * place of dense.  Each pair is applied on its own (theta - lr*v1 - lr*v2 rather than
 * theta - lr*(v1 + v2)); with DGC_FLAG_DETERMINISTIC_ACCUMULATE workers are applied in order,
 * and so they always are by dgc_sparse_sgd_apply_regions (see
 * dgc_decompress_accumulate_regions).
 */
dgc_status dgc_sparse_sgd_apply(dgc_handle* h, float* theta, int64_t n, float learning_rate,
                                int32_t num_payloads, const int32_t* const* idx_ptrs_host,
                                const float* const* val_ptrs_host, const int64_t* pair_counts_host,
                                uint32_t* diag_flags_dev, void* stream);
dgc_status dgc_sparse_sgd_apply_regions(dgc_handle* h, float* theta, float learning_rate,
                                        int32_t num_payloads, const int32_t* const* idx_ptrs_host,
                                        const float* const* val_ptrs_host,
                                        const int32_t* const* count_ptrs_host,
                                        const int64_t* out_offsets_host, void* workspace,
                                        size_t workspace_bytes, void* stream);

/*
 * Wire format (Section 3.1: encode() packs the 32-bit nonzero values and 16-bit run
 * lengths of zeros; the sizes of Tables 3 and 4 count six bytes per entry).
 * Entry e is (runs[e], vals[e]): runs[e] zeros of the flat gradient, then vals[e].  A gap
 * of more than 65535 zeros is bridged by entries (65535, 0.0f), each covering 65536
 * positions (the paper does not say how such gaps are written; this keeps the decoder a
 * plain prefix sum).  Trailing zeros are not encoded.
 *
 * dgc_encode turns one payload in region layout into entries.
 *   idx, val, counts   device, outputs of a dgc_compress call made with
 *                      DGC_FLAG_SORTED_OUTPUT (every region ascending; a region that
 *                      is not raises DGC_DIAG_UNSORTED and is encoded as if adjacent)
 *   runs               device, uint16[entry_capacity]
 *   vals               device, float[entry_capacity]
 *   entry_capacity     dgc_encode_max_entries(pairs) always suffices; entries beyond
 *                      the capacity are dropped and DGC_DIAG_OVERFLOW is raised
 *   num_entries        device, int32: entries the payload needs
 *   workspace          device workspace of this handle (scratch for the prefix sums)
 * Diagnostics are ORed into the workspace's record (dgc_get_diagnostics).
 */
dgc_status dgc_encode_max_entries(const dgc_handle* h, int64_t pairs, int64_t* entries);
dgc_status dgc_encode(dgc_handle* h, const int32_t* idx, const float* val, const int32_t* counts,
                      const int64_t* out_offsets_host, uint16_t* runs, float* vals,
                      int64_t entry_capacity, int32_t* num_entries, void* workspace,
                      size_t workspace_bytes, void* stream);

/*
 * Receive side for encoded payloads: dense[position] += value for every entry of every
 * payload, position = (sum of run + 1 over the entries before it) + its own run.
 *   runs_ptrs_host, vals_ptrs_host   host arrays of num_payloads (1 .. 64) device pointers
 *   entry_counts_host                host, entries in each payload (the receiver knows
 *                                    the message sizes)
 * Entries that land outside [0, n) are skipped and flagged in *diag_flags_dev (may be
 * NULL).  Ordering and DGC_FLAG_DETERMINISTIC_ACCUMULATE as for dgc_decompress_accumulate.
 * Errors: INVALID_ARG, ALIGNMENT, CAPACITY (more entries than a set of n elements can
 * need, or too many payloads), HIP.
 */
dgc_status dgc_decode_accumulate(dgc_handle* h, float* dense, int64_t n, int32_t num_payloads,
                                 const uint16_t* const* runs_ptrs_host,
                                 const float* const* vals_ptrs_host,
                                 const int64_t* entry_counts_host, uint32_t* diag_flags_dev,
                                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * Kernel timing for measurement harnesses.  After dgc_profile_enable the next
 * `max_calls` dgc_compress calls record HIP events on the caller's stream before
 * the norm kernel, after it, after the select kernel, after the streaming kernel
 * and after the emit kernel.  dgc_profile_collect waits for the recorded calls, returns how
 * many there were and the summed durations (milliseconds) of the four kernels, and starts a
 * new batch.  Enabling creates events (a runtime allocation); the hot path itself
 * allocates nothing.  Errors: INVALID_ARG, STATE (collect without enable), HIP.
 */
dgc_status dgc_profile_enable(dgc_handle* h, int32_t max_calls);
dgc_status dgc_profile_collect(dgc_handle* h, int32_t* calls, double* norm_ms, double* select_ms,
                               double* stream_ms, double* emit_ms);
dgc_status dgc_profile_disable(dgc_handle* h);

/*
 * Yardstick for measurement harnesses: one launch of a kernel with the memory traffic of
 * the streaming pass and nothing else (b <- b + a, c <- c + b over the floor(n / 1024)
 * whole tiles of 1024 elements; three arrays read, two written, 20 bytes per element).
 * What it reaches on a given box is the practical ceiling the streaming pass is compared
 * with besides the nominal HBM peak.  a, b, c: device, n floats, 16-byte aligned.
 * groups_per_cu: workgroups (of one wavefront each) a compute unit may hold at a time, 2 to 16;
 * how many bytes per second such a kernel moves depends on it, so a harness tries several and
 * takes the fastest; 0 = as many wavefronts as the streaming pass itself keeps on a compute unit.
 */
dgc_status dgc_profile_stream_ceiling(const float* a, float* b, float* c, int64_t n, int32_t groups_per_cu,
                                      void* stream);

/* Library version, major * 1000 + minor. */
int32_t dgc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DGC_H_ */
