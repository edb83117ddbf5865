/*
 * freeze.h - C ABI of the MI355X (gfx950) Freeze Inference cache-lookup library.
 *
 * The library implements the per-layer approximate cache of the paper
 * "Accelerating Deep Learning Inference via Freezing" (Sec. 2.1 and Sec. 3):
 * a layer's cache is a list of <intermediate output, label> pairs
 * (Pseudocode 1, ConstructCache); a look-up finds the k cached outputs nearest
 * to a query activation, takes a vote over their labels and reports a hit when
 * the agreement reaches the layer's threshold (Sec. 3, the cache look-up API;
 * Pseudocode 1, FreezeInference); a cascade tries the layers in order and
 * forwards only the requests that missed (Pseudocode 1; Sec. 5, "Freeze
 * Inference on GPUs": the batch is rebuilt without the frozen items).
 *
 * Conventions for every entry point
 *  - All data pointers are DEVICE pointers on the current HIP device unless the
 *    parameter comment says "host".  The caller owns every buffer; the library
 *    allocates no device memory and frees nothing it is given.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls only enqueue work on it and return; they never synchronise.
 *    Buffers must stay alive until the enqueued work has finished.
 *  - Return value: FREEZE_OK or a negative error code.  Arguments are checked
 *    on the host before anything is enqueued; on an argument error nothing is
 *    launched and no output is written.  Errors never abort or throw.
 *  - Distances are SQUARED Euclidean distances in fp32.
 *  - Neighbour order is (distance, entry index) ascending: equal distances rank
 *    the lower entry index first.
 *  - Inputs must be finite; the result for NaN/Inf inputs is unspecified.
 *  - A context is plain host state without locks: calls on one context must not overlap in
 *    time on the host (building a layer while another thread looks it up, or two threads
 *    with stage timing enabled).  Look-ups enqueued on different streams may run side by side
 *    on the device when each has its own workspace and outputs; a cache being read must not
 *    be rebuilt until those look-ups have finished.
 */
#ifndef FREEZE_H
#define FREEZE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct freeze_ctx freeze_ctx; /* opaque; host memory; holds per-layer descriptors only */

enum {
    FREEZE_OK = 0,
    FREEZE_EINVAL = -1,     /* null pointer, size or parameter out of range */
    FREEZE_ELAYER = -2,     /* layer index out of range */
    FREEZE_ENOTBUILT = -3,  /* layer has no cache yet */
    FREEZE_EWORKSPACE = -4, /* storage / workspace buffer too small or misaligned */
    FREEZE_EHIP = -5,       /* a HIP runtime call failed (launch error) */
    FREEZE_ESCRATCH = -6    /* freeze_lookup_static: the look-up needs more than FREEZE_STATIC_SCRATCH_BYTES */
};

enum { FREEZE_F32 = 0, FREEZE_BF16 = 1 }; /* element type of the entries handed to freeze_cache_build */

/* Largest k and largest re-scoring width accepted by the look-ups.  The bf16 matrix-core pass
 * keeps FREEZE_MAX_RESCORE candidates per query at most for the exact fp32 re-scoring. */
#define FREEZE_MAX_K 64
#define FREEZE_MAX_RESCORE 64

/* Create / destroy a context with `num_layers` empty layer slots (host-only state). */
int freeze_create(freeze_ctx **out, int num_layers);
int freeze_destroy(freeze_ctx *ctx);

/* Bytes of device memory freeze_cache_build needs in `storage` for an n x d cache
 * (bf16 rows tiled and padded for the matrix cores, fp32 squared norms, labels, a
 * row-major copy of the stored values for exact re-scoring, and the mean vector with its column
 * statistics: about 2x the bf16 size of the cache, 3x when the entries are given in fp32).
 * 0 on invalid arguments. */
size_t freeze_cache_storage_bytes(int64_t n, int64_t d, int entries_dtype);

/*
 * Ingest one layer's cache (Pseudocode 1, ConstructCache: the list of
 * <intermediate output, predicted label> pairs of a layer).
 *   entries  [n, d] row-major, fp32 or bf16 (entries_dtype); the stored values ARE the
 *            cache: distances are measured to exactly these values.
 *   labels   [n] int32, each in [0, num_classes).
 *   storage  caller-owned device buffer of >= freeze_cache_storage_bytes() bytes,
 *            256-byte aligned; everything the look-ups need is copied into it, so
 *            `entries` and `labels` may be released once the stream has run the call.
 *            It must outlive every look-up on this layer.
 * Rebuilding a layer replaces its cache.  Limits: 1 <= n < 2^31 - 512, 1 <= d <= 2^24.
 */
int freeze_cache_build(freeze_ctx *ctx, int layer, const void *entries, int entries_dtype, int64_t n,
                       int64_t d, const int32_t *labels, int32_t num_classes, void *storage,
                       size_t storage_bytes, void *stream);

/*
 * Centring of the caches built from now on with freeze_cache_build (host-side setting of the
 * context; the look-up results do not depend on it, only their speed on caches that sit far from
 * the origin).  The bf16 copy of a cache that the matrix cores rank with, and the bf16 copy of the
 * queries, may be taken relative to the cache's mean vector: distances are unchanged by a common
 * shift, while the ranking key |c|^2 - 2 q.c loses the large common terms whose rounding otherwise
 * hides the differences between neighbours (such queries are still answered exactly, through the
 * slower paths described at freeze_lookup).  The stored values, which distances are measured
 * to, are never altered.
 *   mode 0: never;  1 (default): when the cache's mean dominates its spread, |mean|^2 > 4 x the
 *   summed column variances, decided on the device at build time (mean and variances are taken
 *   over a sample of at most 8,192 evenly spaced entries);  2: always.
 * k-means caches and projections are never centred.
 */
int freeze_set_centring(freeze_ctx *ctx, int mode);

/* Bytes of workspace freeze_lookup needs for a batch of b queries. 0 on invalid arguments. */
size_t freeze_lookup_workspace_bytes(const freeze_ctx *ctx, int layer, int64_t b, int k, int rescore_r);

/*
 * Look up a batch of activations in one layer's cache (Sec. 3, cache look-up
 * API: k nearest neighbours -> k (label, distance) tuples -> label with the most
 * occurrences m_i among the k -> hit decision; Pseudocode 1, FreezeInference).
 *   queries        [b, d] fp32 row-major.
 *   k              neighbours per query, 1 <= k <= min(n, FREEZE_MAX_K).
 *   vote_threshold hit iff the winning label holds >= vote_threshold of the k
 *                  neighbours; 1 <= vote_threshold <= k.
 *   rescore_r      candidates per query kept by the bf16 matrix-core pass and
 *                  re-scored exactly in fp32; 0 = library default (8 for k = 1, 16 for
 *                  k <= 10, 32 for k <= 24, else 64), else k <= rescore_r <= FREEZE_MAX_RESCORE
 *                  (clamped to n).  The width changes the speed, never the result: after
 *                  the re-scoring the library checks, per query, that no entry outside the
 *                  candidates can be nearer than the k-th neighbour found (from the spread
 *                  between coarse keys and exact distances of the candidates themselves, with
 *                  a margin of 8 standard deviations); a query that fails the check is
 *                  re-scored over a wider candidate set (up to 256), and if that fails too it
 *                  is scanned against every entry in fp32 inside the same call.  (With a
 *                  width of 16 or 32 and activations of 4,096 values or more, the last quarter
 *                  of the candidates is itself fetched only when the same check over the
 *                  first three quarters does not already confirm the result.)  A width
 *                  close to k (or data whose bf16 keys cannot tell the neighbours apart:
 *                  clusters far from the origin, k = R) sends more queries down those slower
 *                  paths.
 *   out_labels     [b] int32  winning label (equal counts -> smaller label id).
 *   out_hit        [b] uint8  1 = cache hit.
 *   out_votes      [b] int32  occurrences m of the winning label.
 *   out_nbr_idx    [b, k] int32  entry indices, nearest first.
 *   out_nbr_dist   [b, k] fp32   squared distances, computed as sum (q_i - c_i)^2
 *                  in fp32 (exactly 0 for an entry identical to the query).
 *   workspace      >= freeze_lookup_workspace_bytes() bytes, 256-byte aligned;
 *                  scratch only, contents undefined afterwards.
 * b == 0 is a no-op (the data pointers may then be NULL).  Calls that share a workspace must
 * be ordered on one stream.
 */
int freeze_lookup(freeze_ctx *ctx, int layer, const float *queries, int64_t b, int k, int vote_threshold,
                  int rescore_r, int32_t *out_labels, uint8_t *out_hit, int32_t *out_votes,
                  int32_t *out_nbr_idx, float *out_nbr_dist, void *workspace, size_t workspace_bytes,
                  void *stream);

/*
 * freeze_lookup for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels and results as freeze_lookup, except that the workspace is a buffer of
 * FREEZE_STATIC_SCRATCH_BYTES bytes that lives inside the library's device code (every GPU the
 * library runs on holds one until the process ends).  The call allocates nothing, on the
 * device or through any library.  A look-up whose freeze_lookup_workspace_bytes() exceeds
 * FREEZE_STATIC_SCRATCH_BYTES is refused with FREEZE_ESCRATCH before anything is enqueued
 * (32 MiB covers e.g. 16 queries against 1,000,000 x 512 entries, or 256 queries against
 * 2,000 x 512).  All calls on one GPU share that GPU's buffer, whatever context or stream they
 * use: calls that overlap in time on one GPU race; order them on one stream.  The buffer keeps
 * the last call's contents; nothing in it needs to be zero when a call starts.
 */
#define FREEZE_STATIC_SCRATCH_BYTES (32u << 20)
int freeze_lookup_static(freeze_ctx *ctx, int layer, const float *queries, int64_t b, int k,
                         int vote_threshold, int rescore_r, int32_t *out_labels, uint8_t *out_hit,
                         int32_t *out_votes, int32_t *out_nbr_idx, float *out_nbr_dist, void *stream);

/* Bytes of workspace freeze_lookup_cascade needs. `layers` is a host array. 0 on invalid arguments. */
size_t freeze_cascade_workspace_bytes(const freeze_ctx *ctx, int num_layers, const int *layers, int64_t b,
                                      int k, int rescore_r);

/*
 * Cascaded look-up (Pseudocode 1, FreezeInference; Sec. 5, batch reconstruction):
 * every request is looked up in layers[0]; the requests that miss are compacted
 * (order preserved) and looked up in layers[1], and so on.  No host
 * synchronisation: the number of surviving requests stays on the device.
 *   layers             host array [num_layers] of layer indices, tried in order.
 *   queries_per_layer  host array [num_layers] of device pointers; entry l is
 *                      [b, d_l] fp32; row i of every entry belongs to request i.
 *   vote_thresholds    host array [num_layers].
 *   out_labels         [b] int32  label of the first layer that hit, -1 if none.
 *   out_exit_layer     [b] int32  position (0-based, in `layers`) of that layer, -1 if none
 *                      (the model's own output layer decides; outside this library).
 *   out_hits_per_layer [num_layers] int64  requests frozen at each position.
 */
int freeze_lookup_cascade(freeze_ctx *ctx, int num_layers, const int *layers,
                          const float *const *queries_per_layer, int64_t b, int k,
                          const int *vote_thresholds, int rescore_r, int32_t *out_labels,
                          int32_t *out_exit_layer, int64_t *out_hits_per_layer, void *workspace,
                          size_t workspace_bytes, void *stream);

/*
 * Look-up under the distance-weighted confidence heuristic of Sec. 3: with m_i of the k
 * neighbours carrying label i at distances d_1 .. d_{m_i} (d = square root of the reported
 * squared distance), C_i = (m_i / k) * sum_j 1 / d_j; the label with the largest C_i wins
 * (equal values -> smaller label id) and its C_i is the confidence.  Pseudocode 1,
 * FreezeInference: the look-up is a hit iff confidence > threshold (strict).
 * Arguments as freeze_lookup, except:
 *   conf_threshold  >= 0 (fp32).
 *   out_conf        [b] fp32  confidence of the winning label; +inf when one of its
 *                   neighbours is identical to the query (always a hit).
 *   out_votes       [b] int32 occurrences m of the winning label.
 * The sums are formed in fp64 from the fp32 distances in neighbour order and rounded once.
 */
int freeze_lookup_confidence(freeze_ctx *ctx, int layer, const float *queries, int64_t b, int k,
                             float conf_threshold, int rescore_r, int32_t *out_labels,
                             uint8_t *out_hit, float *out_conf, int32_t *out_votes,
                             int32_t *out_nbr_idx, float *out_nbr_dist, void *workspace,
                             size_t workspace_bytes, void *stream);

/*
 * freeze_lookup_cascade under the confidence rule: position l freezes a request iff its
 * confidence there is > conf_thresholds[l] (host array [num_layers], each >= 0).  Workspace:
 * freeze_cascade_workspace_bytes().
 */
int freeze_lookup_cascade_confidence(freeze_ctx *ctx, int num_layers, const int *layers,
                                     const float *const *queries_per_layer, int64_t b, int k,
                                     const float *conf_thresholds, int rescore_r,
                                     int32_t *out_labels, int32_t *out_exit_layer,
                                     int64_t *out_hits_per_layer, void *workspace,
                                     size_t workspace_bytes, void *stream);

/*
 * Per-layer thresholds from a validation set (Pseudocode 1, ComputeThresholds; Sec. 3.1
 * "Offline Phase"): every validation item is looked up at every layer under the confidence
 * rule, and a layer's threshold is the largest confidence of a look-up whose label differs
 * from the model's own prediction for that item; 0 when no look-up differs.
 *   queries_per_layer  host array [num_layers] of device pointers, [b, d_l] fp32: the
 *                      validation items' intermediate outputs.
 *   model_labels       [b] int32 (device): the label the model predicts for each item.
 *   out_thresholds     [num_layers] fp32 (device).
 * Workspace: freeze_cascade_workspace_bytes().  b == 0 gives thresholds of 0.
 */
int freeze_compute_thresholds(freeze_ctx *ctx, int num_layers, const int *layers,
                              const float *const *queries_per_layer, int64_t b, int k,
                              int rescore_r, const int32_t *model_labels, float *out_thresholds,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * k-means cache (Sec. 4, "k-means"): the points of a layer are clustered and a cache item is
 * a cluster centre with the majority label of its cluster and the share of the cluster that
 * carries it.  freeze_kmeans_build runs `iters` rounds of Lloyd's iterations from the given
 * centres (assignment = the batched look-up of every point against the centres with k = 1,
 * equal distances -> the lower centre; update = mean of the assigned points, summed in point
 * order in fp64 and rounded once to fp32; a cluster that loses all its points keeps its
 * centre, gets label 0 and share 0), then assigns once more for the labels and shares, and
 * leaves `layer` holding that cache.  No host synchronisation.
 *   points        [n, d] fp32 row-major, 16-byte aligned; labels [n] int32 in [0, num_classes),
 *                 num_classes <= 8192.
 *   init_centers  [num_centers, d] fp32; 1 <= num_centers <= n.
 *   storage       >= freeze_kmeans_storage_bytes() bytes, 256-byte aligned; must outlive the
 *                 look-ups on this layer.   workspace  >= freeze_kmeans_workspace_bytes().
 * On such a layer freeze_lookup (k = 1) returns the nearest centre and its majority label, and
 * the confidence entry points (freeze_lookup_confidence, freeze_lookup_cascade_confidence,
 * freeze_compute_thresholds; k must be 1) use the paper's k-means confidence: the majority
 * share over the distance to the centre (zero distance: +inf; an empty cluster: 0).
 * freeze_kmeans_read copies the centres [num_centers, d], majority labels and shares out.
 */
size_t freeze_kmeans_storage_bytes(int64_t num_centers, int64_t d);
size_t freeze_kmeans_workspace_bytes(const freeze_ctx *ctx, int64_t n, int64_t d, int64_t num_centers);
int freeze_kmeans_build(freeze_ctx *ctx, int layer, const float *points, int64_t n, int64_t d,
                        const int32_t *labels, int32_t num_classes, const float *init_centers,
                        int64_t num_centers, int iters, void *storage, size_t storage_bytes,
                        void *workspace, size_t workspace_bytes, void *stream);
int freeze_kmeans_read(freeze_ctx *ctx, int layer, float *out_centers, int32_t *out_majority,
                       float *out_fraction, void *stream);

/*
 * Dimensionality reduction in front of the look-up (Sec. 3: a one-layer network with a hidden
 * layer of 1,024 nodes projects a layer's output before it is cached and looked up):
 * y = W x + bias, optionally through ReLU.  The product runs on the matrix cores in bf16 (x and W
 * rounded to nearest even; a W given in bf16 is taken as it is) with fp32 accumulation.
 * A projection occupies one of the context's slots (look-ups on that slot fail with
 * FREEZE_ENOTBUILT).
 *   weights  [m, d] row-major, fp32 or bf16 (weights_dtype); bias [m] fp32.
 *   storage  >= freeze_projection_storage_bytes() bytes, 256-byte aligned, must outlive the
 *            calls of freeze_project on the slot; build workspace: >= 256 + 4 m bytes.
 *   x        [b, d] fp32, 16-byte aligned;  out [b, m] fp32, 16-byte aligned.
 *   workspace of freeze_project: >= freeze_project_workspace_bytes() bytes.
 * b == 0 is a no-op.
 */
size_t freeze_projection_storage_bytes(int64_t m, int64_t d, int weights_dtype);
int freeze_projection_build(freeze_ctx *ctx, int slot, const void *weights, int weights_dtype, int64_t m,
                            int64_t d, const float *bias, void *storage, size_t storage_bytes,
                            void *workspace, size_t workspace_bytes, void *stream);
size_t freeze_project_workspace_bytes(const freeze_ctx *ctx, int slot, int64_t b);
int freeze_project(freeze_ctx *ctx, int slot, const float *x, int64_t b, int relu, float *out,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * Batch reconstruction on its own (Sec. 5): writes to sel_out the entries
 * sel_in[j] (or j itself when sel_in is NULL) with hit[j] == 0, j < count, in
 * order, and their number to *out_count.
 *   hit       [count] uint8;  sel_in [count] int32 or NULL;  sel_out [count] int32
 *             (hit and sel_out may be NULL when count == 0);
 *   out_count [1] int32.
 */
int freeze_compact_misses(const uint8_t *hit, const int32_t *sel_in, int64_t count, int32_t *sel_out,
                          int32_t *out_count, void *stream);

/*
 * Batch reconstruction of a tensor (Sec. 5, "Freeze Inference on GPUs": the batch is rebuilt
 * after a layer without the frozen items): out[j, :] = x[sel[j], :] for j < *count (or
 * j < max_count when count is NULL), i.e. the next layer's input for the missed requests in
 * miss-list order, as produced by freeze_compact_misses.  No host synchronisation.
 *   x [*, d] fp32;  sel [max_count] int32;  count device int32 or NULL;  out [max_count, d].
 */
int freeze_gather_rows(const float *x, int64_t d, const int32_t *sel, const int32_t *count,
                       int64_t max_count, float *out, void *stream);

/*
 * Counters of how the look-ups of this context were confirmed (measurement aid): while a device
 * array of three uint64 is attached, every look-up adds to it the number of queries whose result was
 * confirmed exact after the first re-scoring [0], after the wider re-scoring [1], and the number
 * redone by the exact scan [2].  The library never clears it.  NULL detaches.
 */
int freeze_lookup_stats_attach(freeze_ctx *ctx, void *counters);

/*
 * Stage timing for benchmarks (measurement aid; the look-up results do not depend on it).
 * While enabled, freeze_lookup records HIP events on its stream around its three stages
 * (query preparation, distance pass, finishing kernels) for up to FREEZE_PROFILE_MAX_CALLS
 * calls; enable = 1: all four stage boundaries; enable = 2: only the two around the distance
 * pass (an event costs a few microseconds of stream time, which shows next to a 0.2 ms look-up;
 * the other two stages then read 0); enable = 3: as 2, for every FREEZE_PROFILE_SAMPLE-th look-up
 * only, starting with the first (for look-ups so short that even two events per call show);
 * enable = 0: off.  freeze_profile_read waits for the recorded
 * events, adds up the stage durations and clears the record.
 *   stage_ms  host array [3]: summed milliseconds of {prep, distance pass, finish}.
 *   calls     host: number of look-ups the sums cover.
 * Events are host-side objects; no device memory is allocated.
 */
#define FREEZE_PROFILE_MAX_CALLS 256
#define FREEZE_PROFILE_SAMPLE 8
int freeze_profile_enable(freeze_ctx *ctx, int enable);
int freeze_profile_read(freeze_ctx *ctx, float *stage_ms, int *calls);
/* Same, per look-up: call_ms is a host array [max_calls][3], filled in call order (a cascade
 * records one look-up per layer); *calls = number of rows written.  Clears the record. */
int freeze_profile_read_calls(freeze_ctx *ctx, float *call_ms, int max_calls, int *calls);

/*
 * Calibration microbenchmarks for benchmarks (they synchronise the device; default stream).
 * freeze_calibrate_mfma: back-to-back bf16 16x16x32 MFMAs from registers on every CU, on
 *   pseudo-random operands (the clock the chip holds under matrix work depends on the data).
 *   scratch        device buffer, 8-byte aligned, >= 2 MiB; contents overwritten.
 *   tflops         host out: sustained dense bf16 rate in TFLOP/s.
 *   shader_mhz     host out: shader clock held under that load, in MHz.
 * freeze_calibrate_hbm_read: reads every byte of `buffer` (device, 16-byte aligned, >= 1 MiB,
 *   initialised by the caller; never written) five times, with non-temporal 16-byte loads, each
 *   workgroup walking a contiguous share.
 *   gbytes_per_s   host out: sustained read rate in GB/s.
 */
int freeze_calibrate_mfma(void *scratch, size_t scratch_bytes, double *tflops, double *shader_mhz);
int freeze_calibrate_hbm_read(const void *buffer, size_t bytes, double *gbytes_per_s);

/* Static description of an error code (host string, never NULL). */
const char *freeze_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* FREEZE_H */
