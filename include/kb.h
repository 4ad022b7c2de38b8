/*
 * kb.h -- C ABI of the MI355X (gfx950) knowledge-base retrieval library.
 *
 * The operation.  The paper's agent keeps a Persistent Knowledge Base of
 * <state, <optimization, score>> entries (Section 3, component list); its State
 * Selector looks up the stored (state, optimization) pairs that fit the kernel's
 * state, the Optimization Selector keeps the top-k of them, and a state that
 * matches nothing is appended (Section 3, the paragraph that walks through one task).  The paper
 * gives that step no numeric form.  This library implements the numeric model
 * of it: entry i has a key vector K_i (row i of an [N, d] matrix) and an
 * optional 64-bit tag; a query is a vector Q_r with an optional 64-bit mask;
 *
 *     score(r, i) = <Q_r, K_i> / (|Q_r| |K_i|)       (0 if either norm is 0)
 *     entry i qualifies for query r  iff  no mask is given or (qmask_r & tag_i) != 0
 *     result(r)   = the k qualifying entries that come first under
 *                   (score descending, index ascending), in that order,
 *                   padded with (index -1, score -inf) when fewer than k qualify.
 *
 * All pointers named *_dev are device (HBM) addresses on the current HIP
 * device; everything else is host memory.  The library never allocates or
 * frees device memory: key storage is borrowed from the caller at kb_create
 * and kb_query works in a caller-provided workspace.  All device work is
 * enqueued on the caller's stream and no call synchronises, except the three
 * that return a device value to the host: kb_query_counters, kb_profile_end
 * and kb_compact.  A handle is not thread-safe.  Calls on one stream are ordered;
 * two kb_query calls may share a workspace only if they are stream-ordered.
 */
#ifndef KB_H
#define KB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kb kb_t; /* opaque, host-side */

typedef enum { KB_F32 = 0, KB_BF16 = 1, KB_FP8_E4M3 = 2 } kb_dtype_t;

typedef enum {
    KB_OK = 0,
    KB_ERR_NULL = 1,           /* a required pointer is NULL */
    KB_ERR_INVALID_ARG = 2,    /* d, capacity, n, Q or k out of range */
    KB_ERR_DTYPE = 3,          /* unknown dtype, or query dtype not allowed for the key dtype */
    KB_ERR_CAPACITY = 4,       /* append would exceed the capacity given at kb_create */
    KB_ERR_NOT_NORMALIZED = 5, /* kb_query while appended rows have no norm yet */
    KB_ERR_NO_TAGS = 6,        /* qmask given but the knowledge base was created without tags */
    KB_ERR_WORKSPACE = 7,      /* workspace NULL, misaligned (256 B) or smaller than kb_query_workspace_bytes */
    KB_ERR_DEVICE = 8          /* a HIP call or kernel launch failed */
} kb_status_t;

#define KB_K_MAX 128 /* largest k accepted by kb_query */

/*
 * Create a knowledge base over caller-owned device storage (Section 3: the
 * store behind the State Selector).  Nothing is copied or launched.
 *   d          vector length; multiple of 32 (KB_F32) or 64 (KB_BF16, KB_FP8_E4M3), <= 16384
 *   key_dtype  element type of keys_dev
 *   capacity   rows the buffers can hold, 1 <= capacity < 2^31
 *   keys_dev       [capacity, d] row-major, 16-byte aligned
 *   row_scale_dev  [capacity] fp32, KB_FP8_E4M3 only (stored value = scale * code); else must be NULL.
 *                  Scales must be finite and > 0; under the cosine they cancel and are not read by queries.
 *   inv_norm_dev   [capacity] fp32, written by kb_normalize (1/|K_i| of the stored codes, 0 for a zero row;
 *                  kb_remove sets the sign bit of a removed entry's word)
 *   tags_dev       [capacity] uint64, or NULL for an untagged knowledge base
 * The buffers must outlive the handle.  Errors: KB_ERR_NULL, KB_ERR_INVALID_ARG, KB_ERR_DTYPE.
 */
kb_status_t kb_create(kb_t **out, int32_t d, kb_dtype_t key_dtype, int64_t capacity, void *keys_dev,
                      float *row_scale_dev, float *inv_norm_dev, uint64_t *tags_dev);

/*
 * Append n rows at index kb_size() .. kb_size()+n-1 (Section 3: a state that the
 * knowledge base does not know yet is added to it).  rows_dev [n, d] in the key dtype, row_scale_dev [n] (fp8 only,
 * else NULL), tags_dev [n] (required iff the KB has tags).  The data is copied
 * device-to-device on `hip_stream`; a source pointer equal to its destination
 * (rows already written in place by the caller) skips that copy.  The new rows
 * are not searchable until kb_normalize.  *first_index_out (host, may be NULL)
 * receives the index of the first new row; it is written only when the call
 * returns KB_OK.  n == 0 is a no-op.
 * Errors: KB_ERR_NULL, KB_ERR_INVALID_ARG (n < 0), KB_ERR_CAPACITY, KB_ERR_DEVICE.
 */
kb_status_t kb_append(kb_t *kb, const void *rows_dev, const float *row_scale_dev, const uint64_t *tags_dev,
                      int64_t n, void *hip_stream, int64_t *first_index_out);

/*
 * Row L2-normalisation as a side scale: for every row appended since the last
 * call, inv_norm[i] = 1 / sqrt(sum_j K_ij^2) in fp32 (0 if the sum is 0); the
 * stored rows are not rewritten.  Cost is proportional to the new rows only.
 * Idempotent.  Errors: KB_ERR_NULL, KB_ERR_DEVICE.
 */
kb_status_t kb_normalize(kb_t *kb, void *hip_stream);

/*
 * Bytes of device workspace that suffice for kb_query and kb_query_sampled with exactly Q queries and this k, at
 * EVERY row count from 0 to the handle's capacity (an upper bound, not the need of the current size: it stays
 * valid while rows are appended) and for every query dtype the handle accepts.  The value depends on the
 * performance knobs of kb_set_tuning: ask again after changing one.  Returns 0 on invalid arguments.
 *
 * kb_query_plan_bytes is the host-side planner behind it: the bytes a query of `kind` (0: kb_query, 1:
 * kb_query_sampled, 2: kb_query with KB_FP8_E4M3 queries, 3: kb_query_sampled with them) needs when the knowledge base holds n rows; 0 when the
 * arguments are invalid or the handle does not take that kind of query.  For every n <= capacity it is at most
 * kb_query_workspace_bytes(kb, Q, k).  No device work.
 */
size_t kb_query_workspace_bytes(const kb_t *kb, int32_t Q, int32_t k);
size_t kb_query_plan_bytes(const kb_t *kb, int64_t n, int32_t Q, int32_t k, int32_t kind);

/*
 * Retrieval (Section 3: State Selector + top-k of the Optimization Selector).
 *   queries_dev [Q, d] row-major, 16-byte aligned; q_dtype must equal the key dtype, except that
 *               KB_FP8_E4M3 keys take KB_BF16 or KB_FP8_E4M3 queries.  fp8 queries are e4m3 codes without a scale (a positive factor per query
 *               row cancels in the cosine); their dot products are formed by the fp8 matrix instruction,
 *               whose 64-term sums are slightly less precise than fp32 (score error up to about 1e-4).
 *   qmask_dev   [Q] uint64, or NULL = no filtering for any query (a zero mask word qualifies nothing)
 *   k           1 .. KB_K_MAX
 *   indices_out_dev [Q, k] int32, scores_out_dev [Q, k] fp32: the result defined at the top of this file,
 *               scores computed as fp32( fp32(dot * inv_norm_i) * inv_norm_q ) with dot accumulated in fp32
 *   workspace_dev   256-byte aligned, at least kb_query_workspace_bytes(kb, Q, k); contents are scratch
 * Results are bit-identical from run to run.  Finite inputs are the caller's responsibility.
 * Errors: KB_ERR_NULL, KB_ERR_INVALID_ARG, KB_ERR_DTYPE, KB_ERR_NOT_NORMALIZED, KB_ERR_NO_TAGS,
 * KB_ERR_WORKSPACE, KB_ERR_DEVICE.  An empty knowledge base returns all padding.
 */
kb_status_t kb_query(kb_t *kb, const void *queries_dev, kb_dtype_t q_dtype, int32_t Q, const uint64_t *qmask_dev,
                     int32_t k, int32_t *indices_out_dev, float *scores_out_dev, void *workspace_dev,
                     size_t workspace_bytes, void *hip_stream);

/*
 * kb_query for callers that cannot allocate device memory or hand over a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical results as
 * kb_query, but the scratch memory is an array of KB_STATIC_SCRATCH_BYTES that is part of the library's device
 * image (one copy per GPU, held until the process ends).  The call allocates and frees nothing; the first call on a
 * device looks the array's address up (make one call before capturing a graph).  A query whose plan needs more than
 * the array holds (kb_query_plan_bytes(kb, kb_size(kb), Q, k, kind) > KB_STATIC_SCRATCH_BYTES: large batches or
 * k on a large knowledge base) returns KB_ERR_WORKSPACE and runs nothing: use kb_query with a workspace then.
 * All calls on one GPU share the array, which keeps the last call's contents; every call resets what it needs
 * zeroed.  Calls that overlap on one GPU (different streams, or threads) race: order them on one stream.
 * kb_query_counters on this scratch is not offered.  Errors: as kb_query.
 */
#define KB_STATIC_SCRATCH_BYTES (32u << 20)
kb_status_t kb_query_static(kb_t *kb, const void *queries_dev, kb_dtype_t q_dtype, int32_t Q, const uint64_t *qmask_dev,
                            int32_t k, int32_t *indices_out_dev, float *scores_out_dev, void *hip_stream);

/*
 * Weighted random selection (Section 3: the Optimization Selector picks its top-k at random, with weights given
 * by the predicted performance gains).  Entry i carries a predicted gain g_i; query r draws
 * k entries WITHOUT replacement from its qualifying entries with probability proportional to
 * g_i * exp(score_ri / temperature).  The draw is the k largest of
 *     key_ri = score_ri / temperature + ln g_i + G_ri,   G_ri = -ln(-ln U_ri)  (standard Gumbel),
 * where U_ri = (upper 23 bits of word (i mod 4) of Philox4x32-10(counter = (i div 4, first_query + r, 0, 0),
 * key = seed) + 1/2) / 2^23, so a result is a pure function of (stored bits, queries, gains, temperature, seed,
 * first_query): bit-identical from run to run and independent of how queries are batched.
 *   gain_dev    [kb_size] fp32 device array, 4-byte aligned, borrowed for the call; an entry with gain <= 0 is
 *               never drawn.  Gains are finite (not checked).
 *   temperature finite, > 0.  seed: any.  first_query >= 0: global number of query row 0.
 *   indices_out_dev [Q, k] int32 and keys_out_dev [Q, k] fp32: drawn entries ordered by (key descending, index
 *               ascending), padded with (-1, -inf) when fewer than k entries qualify.  Keys are computed in fp32
 *               from the fp32 score of kb_query.
 * Everything else (queries, q_dtype, qmask, k, workspace = kb_query_workspace_bytes, stream, errors) as kb_query.
 */
kb_status_t kb_query_sampled(kb_t *kb, const void *queries_dev, kb_dtype_t q_dtype, int32_t Q, const uint64_t *qmask_dev,
                             int32_t k, const float *gain_dev, float temperature, uint64_t seed, int32_t first_query,
                             int32_t *indices_out_dev, float *keys_out_dev, void *workspace_dev, size_t workspace_bytes,
                             void *hip_stream);

/*
 * Row quantisation to E4M3: the storage form of KB_FP8_E4M3 keys (codes + row scale, as kb_create and kb_append
 * take them) and of fp8 queries (codes only), in the numeric model of Section 3's retrieval described at the top
 * of this file.  Independent of any handle.  For every row i of rows_dev [n, d] (KB_F32 or KB_BF16, row-major):
 *     scale_i = max_j |x_ij| / 448 in fp32, or 1 if the row is all zeros
 *     code_ij = the e4m3 code nearest to fp32(x_ij / scale_i): ties to the even code, sign kept, never NaN
 *   codes_out_dev [n, d] bytes; scale_out_dev [n] fp32, or NULL when the scales are not wanted (queries: a
 *   positive factor per row cancels in the cosine).  rows_dev and codes_out_dev 16-byte aligned, not overlapping.
 *   d multiple of 16, 16 .. 16384; 0 <= n < 2^31 (n == 0 is a no-op).  Finite inputs are the caller's responsibility.
 * Errors: KB_ERR_NULL, KB_ERR_DTYPE (rows not KB_F32 / KB_BF16), KB_ERR_INVALID_ARG, KB_ERR_DEVICE.
 */
kb_status_t kb_quantize_rows(const void *rows_dev, kb_dtype_t dtype, int64_t n, int32_t d, void *codes_out_dev,
                             float *scale_out_dev, void *hip_stream);

/*
 * Two-stage retrieval, second stage.  The paper's knowledge base is a hierarchy: states, and below each state its
 * candidate optimizations (Section 3, knowledge-base format and the walk through one task: the state is matched
 * first).  Numeric model: the entries are grouped into clusters, rows of cluster c are
 * [cluster_offsets[c], cluster_offsets[c+1]); a caller first ranks the cluster centroids (an ordinary kb_query on a
 * knowledge base that holds the centroids; its index output is a probe list), then this call returns, for query r,
 * the result kb_query defines, restricted to the entries of the clusters probe[r][0 .. nprobe-1].  Scores are
 * bit-identical to those of kb_query, so the result is exactly the top-k of that subset; how much of the unrestricted
 * top-k it contains (recall) depends on the clustering and on nprobe.
 *   cluster_offsets_dev [n_clusters + 1] int64, non-decreasing, within [0, kb_size]; a cluster may be empty
 *   probe_dev  [Q, nprobe] int32; entries outside [0, n_clusters) (the -1 padding of a result list) are skipped, a
 *              cluster named twice counts once;  1 <= nprobe <= 64,  1 <= Q <= 65535
 *   queries, q_dtype, qmask, k, outputs, stream: as kb_query (fp8 queries are accepted for any d here); removed
 *   entries are never returned
 *   workspace_dev  256-byte aligned, at least kb_query_probe_workspace_bytes(kb, Q, k, nprobe) (0 on invalid arguments)
 * Cost is proportional to the rows of the probed clusters, not to kb_size: meant for small batches.
 * Errors: as kb_query.
 */
size_t kb_query_probe_workspace_bytes(const kb_t *kb, int32_t Q, int32_t k, int32_t nprobe);
kb_status_t kb_query_probe(kb_t *kb, const void *queries_dev, kb_dtype_t q_dtype, int32_t Q, const uint64_t *qmask_dev,
                           int32_t k, const int64_t *cluster_offsets_dev, int32_t n_clusters, const int32_t *probe_dev,
                           int32_t nprobe, int32_t *indices_out_dev, float *scores_out_dev, void *workspace_dev,
                           size_t workspace_bytes, void *hip_stream);

/*
 * Revision of predicted gains: the numeric side of the paper's ParameterUpdate step (Section 3; the last step of
 * the outer loop of Algorithm 2 rewrites the knowledge base from what the rollouts measured).  For j = 0 .. m-1:
 *     i = indices[j];   gain[i] <- gain[i] + alpha * (values[j] - gain[i])      (fp32: one subtraction, one fma)
 * an exponential moving average towards the observed gain; alpha = 1 stores values[j] itself.  An index outside [0, n) (the -1
 * padding of a result list) is skipped.  Indices must be distinct within a call (otherwise one of the pairs wins).
 *   gain_dev [n] fp32 (the array kb_query_sampled takes), indices_dev [m] int32, values_dev [m] fp32, 0 <= alpha <= 1.
 * Errors: KB_ERR_NULL, KB_ERR_INVALID_ARG (n or m negative, alpha outside [0, 1] or NaN, misaligned), KB_ERR_DEVICE.
 */
kb_status_t kb_update_gain(float *gain_dev, int64_t n, const int32_t *indices_dev, const float *values_dev, int64_t m,
                           float alpha, void *hip_stream);

/*
 * Removal (knowledge-base management; the paper's conclusion names it as future work).  The m entries keep their
 * rows and indices, kb_size does not change, but no kb_query / kb_query_sampled enqueued afterwards returns them.
 * The mark is the sign bit of the entry's inv_norm word.  Indices outside [0, kb_size) are skipped; repeats are
 * harmless.  Rows appended but not yet normalised cannot be removed (KB_ERR_NOT_NORMALIZED).
 * Errors: KB_ERR_NULL, KB_ERR_INVALID_ARG, KB_ERR_NOT_NORMALIZED, KB_ERR_DEVICE.
 */
kb_status_t kb_remove(kb_t *kb, const int32_t *indices_dev, int64_t m, void *hip_stream);

/*
 * Compaction: copies the entries of `src` that have not been removed, in their order, into the EMPTY knowledge
 * base `dst` (same d, dtype and taggedness, separate storage, capacity >= the number of live entries), with their
 * norms, scales and tags; dst is then normalised and ready for queries, src is unchanged.
 *   gain_src_dev / gain_dst_dev  optional per-entry fp32 array carried along ([kb_size(src)] -> [live]); both or neither
 *   index_map_out_dev            optional [kb_size(src)] int32: new index of each old entry, -1 if removed
 *   workspace_dev                256-byte aligned, at least kb_compact_workspace_bytes(src)
 *   live_out                     host, optional: number of entries copied (= kb_size(dst) afterwards)
 * This call SYNCHRONISES `hip_stream` once (the live count decides the capacity check and dst's size), so it cannot
 * be captured in a graph.  Errors: KB_ERR_NULL, KB_ERR_INVALID_ARG (shape mismatch, dst not empty, shared storage),
 * KB_ERR_DTYPE, KB_ERR_NOT_NORMALIZED, KB_ERR_WORKSPACE, KB_ERR_CAPACITY (dst too small; nothing was written),
 * KB_ERR_DEVICE.
 */
size_t kb_compact_workspace_bytes(const kb_t *kb);
kb_status_t kb_compact(kb_t *src, kb_t *dst, const float *gain_src_dev, float *gain_dst_dev, int32_t *index_map_out_dev,
                       void *workspace_dev, size_t workspace_bytes, void *hip_stream, int64_t *live_out);

/*
 * Self-check of a property the main pass of kb_query_sampled relies on (Section 3, Optimization Selector: the
 * weighted random choice): it rejects most (query, entry) pairs by comparing the random generator's word with a bound,
 * without computing the pair's key, which is exact as long as the noise G = -ln(-ln U) that the device computes is a
 * non-decreasing function of the 23 bits of the word that make U.  The call enqueues on `hip_stream` a kernel that
 * evaluates G for all 2^23 values and writes out_dev[0] = values whose G is below that of the value before (0 on a
 * device the library is valid for), out_dev[1] = values looked at (2^23).  `out_dev`: device memory, 2 x int64, the
 * caller's; read it after synchronising the stream.  Errors: KB_ERR_NULL, KB_ERR_DEVICE.
 */
kb_status_t kb_check_draw_noise(int64_t *out_dev, void *hip_stream);

/*
 * Diagnostics of the most recent kb_query that used `workspace_dev`: synchronises `hip_stream`, then copies
 * out[0] = candidates that passed the threshold filter (all queries), out[1] = queries resolved by the
 * exhaustive per-query path, out[2] = keys scored by the sampling pass, out[3] = workgroups of the scan (a query
 * that took the small-knowledge-base path reports 0, 0, 0 and its workgroups).
 * `out` is host memory, 4 x int64.  Errors: KB_ERR_NULL, KB_ERR_DEVICE.
 */
kb_status_t kb_query_counters(const kb_t *kb, const void *workspace_dev, int64_t *out, void *hip_stream);

/*
 * Performance knobs; they never change results.  Unknown names return KB_ERR_INVALID_ARG.
 *   "sample_keys"   keys scored by the sampling pass (0 = automatic)
 *   "scan_config"   tile configuration of the scan kernel (0 = automatic)
 *   "wg_per_cu"     resident scan workgroups per compute unit (0 = automatic)
 *   "small_path"    1 (default): a knowledge base of at most 16384 rows, queried with a small batch and no other knob
 *                   set, is scored whole by two launches (no sampling pass, no candidate lists); 0: always the
 *                   scan pipeline.  Both produce the same bits.
 *   "profile_stride" of a kb_profile_begin session, every value-th scan launch is timed: launch value/2 of each run of
 *                   `value` launches (0 or 1: every one).  A timed
 *                   launch costs the stream about 12 us of idle time around it; a stride spreads the timed launches
 *                   evenly over the session and keeps that cost small.
 */
kb_status_t kb_set_tuning(kb_t *kb, const char *name, int64_t value);

/*
 * Kernel timing for roofline reports.  After kb_profile_begin, each kb_query attaches a HIP event pair to the
 * dispatch of its main scan kernel (on the small-knowledge-base path an event pair is recorded around the kernel
 * that scores the rows), up to max_calls timed queries, 1..4096; later ones are not timed (see "profile_stride"
 * above to time every n-th query only).  The pair travels with the kernel's own dispatch packet; a timed dispatch is
 * still preceded and followed by a few microseconds in which the stream runs nothing.
 * kb_profile_end synchronises `hip_stream`, writes the summed duration of the timed scan launches in milliseconds and
 * their number, destroys the events and stops recording.
 * Errors: KB_ERR_NULL, KB_ERR_INVALID_ARG (bad max_calls, or end without begin), KB_ERR_DEVICE.
 */
kb_status_t kb_profile_begin(kb_t *kb, int32_t max_calls);
kb_status_t kb_profile_end(kb_t *kb, void *hip_stream, double *scan_ms_total, int32_t *calls);

int64_t kb_size(const kb_t *kb);         /* rows appended so far; -1 if kb is NULL */
kb_status_t kb_destroy(kb_t *kb);        /* frees the host struct only */
const char *kb_status_string(kb_status_t s);

#ifdef __cplusplus
}
#endif
#endif /* KB_H */
