/*
 * dp.h -- C ABI of the MI355X (gfx950) Double-P decode-attention library.
 *
 * One decode step, one layer, of hierarchical top-p sparse attention over a
 * clustered KV cache (paper Sec. 4.2-4.4):
 *   stage 1  size-weighted centroid scoring                 (Eq. 3, Eq. 5, Eq. 6)
 *   stage 2  first top-p over clusters, second top-p that splits the retained
 *            clusters into "exact" and "approximated"        (Eq. 7, Sec. 4.3)
 *   stage 3  attention over the tokens of the exact clusters plus one
 *            size-weighted centroid pseudo-token per approximated cluster,
 *            with one shared normaliser                      (Eq. 8, Eq. 9)
 *
 * Conventions for every entry point
 *   - Plain C linkage, no exceptions, no torch types.
 *   - Every pointer inside dp_problem and every buffer argument is a DEVICE
 *     pointer owned by the caller, unless the comment says "host".  dp_problem
 *     itself is a host struct read during the call only.
 *   - Calls enqueue work on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and return without synchronising.  Nothing is allocated
 *     or freed; the library keeps no state between calls that changes a result
 *     (it remembers per process how many workgroups of a kernel the device
 *     holds, asked from the runtime once, and dp_decode_attention_static owns a
 *     scratch array).  Inputs are never written.  Two calls that share a workspace must be ordered by the caller.
 *   - Errors that can be detected on the host (null pointers, bad shapes, p out
 *     of range, workspace too small, unsupported head_dim) are returned before
 *     anything is launched.  Device data (offsets, sizes, ids) is NOT validated:
 *     out-of-range values there are undefined behaviour.
 *   - A "head" is a (sequence b, query head h) pair, index b*n_q_heads + h.  It
 *     reads KV segment seg = b*n_kv_heads + h/(n_q_heads/n_kv_heads).
 *   - Cluster ids in sel_ids are segment-local (0 .. Kc_seg-1).
 */
#ifndef DP_H
#define DP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  DP_OK = 0,
  DP_ERR_INVALID_ARG = -1,         /* null pointer, non-positive shape, p outside its domain        */
  DP_ERR_UNSUPPORTED = -2,         /* head_dim != 128, n_q_heads/n_kv_heads > 16, unknown dtype     */
  DP_ERR_WORKSPACE_TOO_SMALL = -3, /* workspace_bytes < dp_workspace_bytes(problem)                 */
  DP_ERR_HIP = -4,                 /* a HIP runtime call failed (launch error)                      */
  DP_ERR_TOO_LARGE = -5            /* dp_decode_attention_static: dp_workspace_bytes(problem) > DP_STATIC_SCRATCH_BYTES */
} dp_status;

typedef enum { DP_BF16 = 0, DP_F32 = 1 } dp_dtype;

/* Second top-p reading.  Default: the exact set is the shortest prefix of the
 * score order whose estimated mass reaches p2 * M1, M1 being the mass kept by
 * the first top-p (a top-p over the retained set).  With this flag the
 * threshold is min(p2, M1): p2 measured on the whole distribution. */
#define DP_FLAG_P2_ABSOLUTE 1u
/* dp_decode_attention runs the split decode of stage 3 inside the selection launch (two kernel launches per step)
 * when a step serves at most 128 heads.  With this flag it always uses a separate decode launch (three launches),
 * as it does for all other steps: faster by about a tenth when every head of the step is flat (a caller who knows
 * may say so), slower when most heads are peaked.  Same sets; the outputs may differ in the last bits (the rows of
 * a head are split into partial results differently). */
#define DP_FLAG_SEPARATE_DECODE_LAUNCH 2u

typedef struct {
  int32_t batch, n_kv_heads, n_q_heads, head_dim; /* n_q_heads % n_kv_heads == 0; head_dim == 128 */
  const void *q;                  /* bf16 [batch, n_q_heads, head_dim]                                  */
  const void *k_cache;            /* bf16 [total_rows, head_dim]; a cluster's rows are consecutive      */
  const void *v_cache;            /* bf16 [total_rows, head_dim]; same row order as k_cache             */
  const int64_t *seg_row_base;    /* [batch*n_kv_heads]    first cache row of each segment              */
  const int32_t *seg_cluster_ptr; /* [batch*n_kv_heads+1]  CSR: clusters of seg are [ptr[seg],ptr[seg+1]) */
  const int32_t *cluster_offsets; /* [total_clusters] first row of the cluster, relative to seg_row_base */
  const int32_t *cluster_sizes;   /* [total_clusters] s_i >= 0; a cluster with s_i == 0 is never selected */
  const void *k_centroids;        /* bf16 [total_clusters, head_dim]  C_i: mean key of the cluster      */
  const void *v_centroids;        /* bf16 [total_clusters, head_dim]  mean value (Eq. 2), NOT the sum   */
  int32_t total_clusters;         /* host-known: seg_cluster_ptr[batch*n_kv_heads]                      */
  int32_t max_clusters_per_seg;   /* host-known upper bound on ptr[seg+1]-ptr[seg]                      */
  int32_t max_rows_per_seg;       /* host-known upper bound on the rows (tokens) of one segment         */
  float sm_scale;                 /* logit scale; 0 => 1/sqrt(head_dim)                                 */
  uint32_t flags;                 /* DP_FLAG_*                                                          */
  const uint8_t *cluster_flags;   /* [total_clusters] DP_CLUSTER_* bits per cluster, or NULL (none set) */
} dp_problem;

/* A pinned cluster holds tokens that are always attended exactly: the sink and
 * sliding-window tokens that the paper's runs keep dense at every layer while
 * the sparse selection sees only the remaining tokens (Sec. 5.1).  Stage 2
 * (dp_topp_select, dp_topk_select and the one-call entry points) ignores the
 * logit of a pinned cluster: it takes no part in the softmax over clusters,
 * the thresholds or a budget, and it is always a member of the exact list
 * (counted in n_exact, n_retained, n_exact_tokens) unless it is empty.
 * dp_score_centroids still writes its Eq. 3 / Eq. 5 logit; dp_sparse_decode
 * and dp_dense_decode do not read the flags. */
#define DP_CLUSTER_PINNED 1u

/* Host-only.  Bytes of device workspace that dp_sparse_decode and
 * dp_decode_attention need for this problem (depends on the shape fields and
 * the three host-known bounds only).  Returns 0 for an invalid problem. */
size_t dp_workspace_bytes(const dp_problem *problem);

/* Number of floats in the logits buffer: (n_q_heads/n_kv_heads) * total_clusters. */
size_t dp_logits_count(const dp_problem *problem);

/* Stage 1 (Eq. 3, 5, 6 before normalisation).  For head (b, h), j = h % G,
 * G = n_q_heads/n_kv_heads, and cluster i of its segment:
 *   logits[G*ptr[seg] + j*Kc_seg + i] = sm_scale * (q[b,h] . C_i) + ln(s_i)   (fp32; -inf if s_i == 0)
 * i.e. one contiguous fp32 row of Kc_seg logits per head.  Each centroid row is
 * read once and scored against the G query heads that share it. */
dp_status dp_score_centroids(const dp_problem *problem, float *logits, void *stream);

/* dp_score_centroids for measurement: start_event / stop_event (hipEvent_t passed as void*, created by the
 * caller with timing enabled, either may be NULL) receive the begin and end timestamps of the scoring kernel
 * itself (not of the gap before it), so hipEventElapsedTime(start, stop) after the stream has drained is the
 * kernel's duration.  Same result and errors as dp_score_centroids. */
dp_status dp_score_centroids_timed(const dp_problem *problem, float *logits, void *stream, void *start_event,
                                   void *stop_event);

/* Stage 2 (Eq. 6 softmax, Eq. 7 first top-p, Sec. 4.3 second top-p).  Per head:
 * clusters are ordered by logit descending, ties by lower cluster index; the
 * retained set is the shortest prefix whose softmax mass reaches p1 (all
 * non-empty clusters when p1 >= 1); the exact set is the shortest prefix that
 * reaches the second threshold (see DP_FLAG_P2_ABSOLUTE; p2 >= 1 => every
 * retained cluster, p2 == 0 => none).  Domain 0 < p1 <= 1, 0 <= p2 <= 1.
 * Outputs (device):
 *   sel_ids  int32 [batch*n_q_heads, max_clusters_per_seg]: per head the exact
 *            ids in ascending order, then the approximated ids in ascending order;
 *   n_exact, n_retained, n_exact_tokens  int32 [batch*n_q_heads]
 *            (n_exact_tokens = sum of s_i over the exact set).
 * Masses are accumulated in 2^-40 fixed point, so the result is independent of
 * thread scheduling (bitwise reproducible). */
dp_status dp_topp_select(const dp_problem *problem, const float *logits, float p1, float p2, int32_t *sel_ids,
                         int32_t *n_exact, int32_t *n_retained, int32_t *n_exact_tokens, void *stream);

/* Stage 3 (Eq. 8, Eq. 9) for caller-given sets in the dp_topp_select format
 * (exact ids first, n_exact of them, then n_retained - n_exact approximated
 * ids; ids unique, each cluster non-empty).  n_exact_tokens is recomputed, the
 * argument may be NULL.
 *   out  [batch, n_q_heads, head_dim] of out_dtype;  lse (nullable) fp32
 *   [batch*n_q_heads] = ln of the shared normaliser Z~.  A head with an empty
 *   retained set gets out = 0, lse = -inf.
 * workspace: at least dp_workspace_bytes(problem) bytes, 256-byte aligned. */
dp_status dp_sparse_decode(const dp_problem *problem, const int32_t *sel_ids, const int32_t *n_exact,
                           const int32_t *n_retained, const int32_t *n_exact_tokens, void *out, dp_dtype out_dtype,
                           float *lse, void *workspace, size_t workspace_bytes, void *stream);

/* A/B variant: selection per GQA group.  The paper states the method for a
 * single query; its model has groups of 4 query heads per KV head (Sec. 5.1) and
 * the text does not say whether the two top-p sets are taken per query head or
 * per group.  The library's path takes them per head.  This entry point takes
 * them per head (exactly as dp_topp_select) and then lets EVERY head of a group
 * attend (Eq. 8, Eq. 9) over the union of the group's sets:
 *   exact(group)  = union over the heads h of C_exact(h)
 *   approx(group) = (union over h of C_p1(h)) minus exact(group)
 * so that a K / V row is read once per group.  Each head attends a superset of
 * its own selection, so the output differs from dp_decode_attention's (it lies
 * between it and dense attention).  Outputs besides out / lse (lse nullable):
 *   union_ids    int32 [batch*n_kv_heads, max_clusters_per_seg]  per segment:
 *                exact ids ascending, then approximated ids ascending (segment-local)
 *   n_exact_u    int32 [batch*n_kv_heads]
 *   n_retained_u int32 [batch*n_kv_heads]   exact + approximated
 * all device, caller-owned.  Workspace as dp_decode_attention.  DP_ERR_UNSUPPORTED
 * for more than 65536 clusters per segment. */
dp_status dp_group_union_decode_attention(const dp_problem *problem, float p1, float p2, void *out,
                                          dp_dtype out_dtype, float *lse, int32_t *union_ids, int32_t *n_exact_u,
                                          int32_t *n_retained_u, void *workspace, size_t workspace_bytes,
                                          void *stream);

/* A/B variant of dp_sparse_decode in the structure the paper describes for its
 * own kernels (Sec. 4.4): the K / V rows of every head's exact clusters are first
 * copied into a contiguous per-head buffer (k_buf, v_buf: bf16
 * [batch*n_q_heads, rows_cap, head_dim], device), and the weighted flash-decode
 * then reads that buffer instead of the cache (centroid rows are still read in
 * place; a head with more than rows_cap exact rows is not copied and is read in
 * place).  Same arithmetic in the same order, hence the same output bits as
 * dp_sparse_decode; it exists to time the two designs against each other. */
dp_status dp_sparse_decode_gathered(const dp_problem *problem, const int32_t *sel_ids, const int32_t *n_exact,
                                    const int32_t *n_retained, void *out, dp_dtype out_dtype, float *lse,
                                    void *k_buf, void *v_buf, int32_t rows_cap, void *workspace,
                                    size_t workspace_bytes, void *stream);

/* Stages 1-3 in one call (logits and id lists live in the workspace).  n_exact,
 * n_retained, n_exact_tokens (int32 [batch*n_q_heads]) and lse are optional
 * outputs (NULL to skip). */
dp_status dp_decode_attention(const dp_problem *problem, float p1, float p2, void *out, dp_dtype out_dtype,
                              float *lse, int32_t *n_exact, int32_t *n_retained, int32_t *n_exact_tokens,
                              void *workspace, size_t workspace_bytes, void *stream);

/* Host-only.  Kernel launches that one dp_decode_attention call enqueues for this problem: scoring, selection (with
 * the attention of heads of few rows), and the split decode either inside the selection launch or as launches of
 * its own, one per 1024 heads (see DP_FLAG_SEPARATE_DECODE_LAUNCH).  0 for an invalid problem or one without
 * clusters. */
int32_t dp_decode_attention_launches(const dp_problem *problem);

/* dp_decode_attention for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same computation, same kernels and same results as
 * dp_decode_attention; the workspace is a device array of DP_STATIC_SCRATCH_BYTES
 * that is part of the library's code object (each GPU the library runs on holds
 * its own copy until the process ends).  The call allocates and frees nothing
 * and records no memset: every counter in the scratch is cleared by the kernels
 * that use it.  The first call on a device looks the array's address up
 * (hipGetSymbolAddress, with that device current); make that call outside a
 * graph capture.
 *   DP_ERR_TOO_LARGE  dp_workspace_bytes(problem) > DP_STATIC_SCRATCH_BYTES (checked on
 *                     the host before anything is launched; 16 MiB holds batch 1 x
 *                     32 query heads x 8192 clusters per KV head at 131072 tokens)
 * All calls on one GPU share that GPU's array and find the previous call's
 * contents in it: calls that overlap on one GPU (two streams, two threads) race;
 * calls on one stream, or otherwise ordered by the caller, do not. */
#define DP_STATIC_SCRATCH_BYTES (16u << 20)
dp_status dp_decode_attention_static(const dp_problem *problem, float p1, float p2, void *out, dp_dtype out_dtype,
                                     float *lse, int32_t *n_exact, int32_t *n_retained, int32_t *n_exact_tokens,
                                     void *stream);

/* dp_decode_attention for measurement: events is a HOST array of 6 hipEvent_t
 * (passed as void*, created by the caller with timing enabled, any may be
 * NULL): {score begin, score end, select begin, select end, decode begin,
 * decode end}.  Each pair receives the begin and end timestamps of that kernel
 * itself, so after the stream has drained hipEventElapsedTime of a pair is the
 * kernel's duration inside the one-call path and the time between pairs is the
 * gap between the kernels.  Same result and errors as dp_decode_attention
 * (without the optional count outputs). */
dp_status dp_decode_attention_timed(const dp_problem *problem, float p1, float p2, void *out, dp_dtype out_dtype,
                                    float *lse, void *workspace, size_t workspace_bytes, void *stream,
                                    void *const *events);

/* A/B variant of dp_topp_select in the structure the paper describes for its own
 * top-p kernel (Sec. 4.4): the cluster scores of a head are sorted first and the
 * two cuts are taken by a prefix sum along the sorted order.  Same masses, same
 * order, same tie-break, hence the same outputs as dp_topp_select; it exists to
 * time the two designs against each other and nothing in the library calls it.
 * DP_ERR_UNSUPPORTED for more than 8192 clusters per segment or with
 * cluster_flags set. */
dp_status dp_topp_select_sorted(const dp_problem *problem, const float *logits, float p1, float p2, int32_t *sel_ids,
                                int32_t *n_exact, int32_t *n_retained, int32_t *n_exact_tokens, void *stream);

/* Stage 2 with a fixed budget in place of the two thresholds: the fixed top-k
 * cluster retrieval of the cluster-based baseline the paper compares with
 * (Sec. 5.1 "Baselines").  Same order as dp_topp_select (logit descending,
 * ties by lower cluster index, empty clusters never selected): the first
 * min(k_retained, non-empty clusters) clusters are retained and the first
 * min(k_exact, that) of them are exact.  k_retained == 0 selects nothing.
 * Outputs as dp_topp_select.  DP_ERR_INVALID_ARG for a negative budget. */
dp_status dp_topk_select(const dp_problem *problem, const float *logits, int32_t k_retained, int32_t k_exact,
                         int32_t *sel_ids, int32_t *n_exact, int32_t *n_retained, int32_t *n_exact_tokens,
                         void *stream);

/* dp_decode_attention with the selection rule of dp_topk_select. */
dp_status dp_budget_decode_attention(const dp_problem *problem, int32_t k_retained, int32_t k_exact, void *out,
                                     dp_dtype out_dtype, float *lse, int32_t *n_exact, int32_t *n_retained,
                                     int32_t *n_exact_tokens, void *workspace, size_t workspace_bytes, void *stream);

/* Dense attention (Sec. 2.1, Eq. 1) over every token of each head's KV segment:
 * the full-attention baseline of the paper's efficiency comparison (Sec. 5.3).
 * The tokens of segment seg are the cache rows [seg_row_base[seg],
 * seg_row_base[seg] + seg_rows[seg]); seg_rows is a DEVICE array, int32
 * [batch*n_kv_heads], each entry <= max_rows_per_seg (larger values are
 * clamped to it).  The cluster arrays of the problem are not read and may be
 * NULL.  K/V rows are read once per KV head and scored against all query heads
 * of the GQA group (any group size).  out, lse, workspace as dp_sparse_decode;
 * a segment without rows gives out = 0, lse = -inf. */
dp_status dp_dense_decode(const dp_problem *problem, const int32_t *seg_rows, void *out, dp_dtype out_dtype,
                          float *lse, void *workspace, size_t workspace_bytes, void *stream);

/* ---- prefill side: the cluster-contiguous cache and its metadata (Sec. 4.1, Eq. 2) ---- */

/* K / V of the context in token order with one cluster id per token (the result
 * of the clustering step, which is not part of this library).  Segment seg owns
 * rows [seg_row_base[seg], seg_row_base[seg] + seg_rows[seg]) of k_tokens,
 * v_tokens, assignment AND of the output cache, and clusters
 * [seg_cluster_ptr[seg], seg_cluster_ptr[seg+1]).  All pointers are device
 * pointers; the three bounds are host-known. */
typedef struct {
  int32_t n_seg;                  /* batch * n_kv_heads                                                  */
  int32_t head_dim;               /* 128                                                                 */
  const void *k_tokens;           /* bf16 [total_rows, head_dim], token order                            */
  const void *v_tokens;           /* bf16 [total_rows, head_dim]                                         */
  const int32_t *assignment;      /* [total_rows] segment-local cluster id of each token                 */
  const int64_t *seg_row_base;    /* [n_seg]                                                             */
  const int32_t *seg_rows;        /* [n_seg] tokens of each segment (clamped to max_rows_per_seg)        */
  const int32_t *seg_cluster_ptr; /* [n_seg+1]                                                           */
  int32_t total_clusters;         /* seg_cluster_ptr[n_seg]                                              */
  int32_t max_clusters_per_seg;   /* upper bound on ptr[seg+1]-ptr[seg]                                  */
  int32_t max_rows_per_seg;       /* upper bound on seg_rows[seg]                                        */
} dp_prefill;

/* Host-only.  Device workspace dp_build_cluster_cache needs (per segment and
 * 1024-token block one int32 per cluster, plus 6 bytes per token); 0 for an
 * invalid description. */
size_t dp_build_workspace_bytes(const dp_prefill *in);

/* Builds what the decode entry points read (the dp_problem fields of the same
 * names): clusters laid out in index order, the tokens of a cluster in token
 * order (a stable counting sort by cluster id):
 *   k_cache, v_cache   bf16 [total_rows, head_dim]   the rows, cluster-contiguous
 *   cluster_sizes      int32 [total_clusters]        s_i = |T_i|
 *   cluster_offsets    int32 [total_clusters]        exclusive prefix of the sizes per segment
 *   k_centroids        bf16 [total_clusters, d]      C_i: mean key of the cluster
 *   v_centroids        bf16 [total_clusters, d]      V-bar_i = V^Sigma_i / s_i (Eq. 2)
 *   v_sums (nullable)  fp32 [total_clusters, d]      V^Sigma_i (Eq. 2)
 *   token_row (nullable) int32 [total_rows]          segment-relative cache row of each token, -1 if left out
 * Means are fp64 sums in row order divided by s_i and rounded ONCE to bf16 (ties
 * to even); an empty cluster gets zero rows.  A token whose id is outside
 * [0, clusters of its segment) is left out of the cache.  Bitwise reproducible.
 * The outputs must not alias the inputs.  workspace: dp_build_workspace_bytes,
 * 256-byte aligned.  DP_ERR_UNSUPPORTED: head_dim != 128 or more than 65536
 * clusters in a segment (in->max_clusters_per_seg). */
dp_status dp_build_cluster_cache(const dp_prefill *in, void *k_cache, void *v_cache, int32_t *cluster_offsets,
                                 int32_t *cluster_sizes, void *k_centroids, void *v_centroids, float *v_sums,
                                 int32_t *token_row, void *workspace, size_t workspace_bytes, void *stream);

/* Assignment step of the k-means clustering of the keys (Sec. 4.1): every token
 * of segment seg goes to the nearest of the segment's centroids,
 *   assignment[row] = argmax_c ( x . c - |c|^2 / 2 )   (= argmin_c |x - c|^2),
 * the lower index on a tie; -1 if the segment has no centroid.  bf16 operands,
 * fp32 accumulation on the matrix cores (two centroids whose scores differ by
 * less than fp32 rounding of a 128-term sum may swap against exact arithmetic).
 * Uses in->k_tokens, seg_row_base, seg_rows, seg_cluster_ptr and the three
 * bounds; in->v_tokens and in->assignment are not read.
 *   centroids   bf16 [total_clusters, head_dim]  (device)
 *   assignment  int32 [total_rows]               (device, written)
 *   best_score  fp32 [total_rows], nullable: the winning x . c - |c|^2 / 2
 * With dp_build_cluster_cache (which recomputes the centroids as the cluster
 * means) this is one Lloyd iteration; initial centroids and the iteration count
 * are the caller's.  workspace: dp_kmeans_workspace_bytes, 256-byte aligned. */
size_t dp_kmeans_workspace_bytes(const dp_prefill *in);
dp_status dp_kmeans_assign(const dp_prefill *in, const void *centroids, int32_t *assignment, float *best_score,
                           void *workspace, size_t workspace_bytes, void *stream);

/* k-means over the key vectors of every segment as a procedure (Sec. 4.1 names
 * k-means and fixes neither the initial centroids, nor the number of iterations,
 * nor the fate of a cluster that loses its tokens; the choices below are this
 * library's).  Lloyd's iteration, n_iters rounds on the device, no host
 * synchronisation:
 *   assignment  dp_kmeans_assign's rule on the current centroids;
 *   update      centroid = mean key of the cluster's tokens (fp64 sums in token
 *               order, rounded once to bf16, as dp_build_cluster_cache does); a
 *               cluster without tokens keeps its centroid.
 * init: DP_KMEANS_INIT_GIVEN     centroids holds the initial centroids;
 *       DP_KMEANS_INIT_STRIDED   centroid c of a segment with n tokens and kc
 *                                clusters starts as the key of token
 *                                floor(c * n / kc) (a zero row if n == 0).
 *   centroids   bf16 [total_clusters, head_dim] (device, read and written): on
 *               return, the centroids after the last update
 *   assignment  int32 [total_rows] (device, written; may be null if n_iters == 0):
 *               the last round's assignment, made with the centroids BEFORE that
 *               round's update.  dp_build_cluster_cache on it gives a cache whose
 *               key centroids equal `centroids` for every non-empty cluster.
 *   best_score  fp32 [total_rows], nullable: as dp_kmeans_assign, last round
 * in->v_tokens and in->assignment are not read.  n_iters == 0 only initialises.
 * workspace: dp_kmeans_fit_workspace_bytes, 256-byte aligned.  Errors as the two
 * steps'; DP_ERR_INVALID_ARG also for n_iters < 0 or an unknown init. */
#define DP_KMEANS_INIT_GIVEN 0u
#define DP_KMEANS_INIT_STRIDED 1u
size_t dp_kmeans_fit_workspace_bytes(const dp_prefill *in);
dp_status dp_kmeans_fit(const dp_prefill *in, void *centroids, int32_t n_iters, uint32_t init, int32_t *assignment,
                        float *best_score, void *workspace, size_t workspace_bytes, void *stream);

/* Where dp_decode_attention keeps its intermediate results inside the
 * workspace (byte offsets; host-only, for inspection by tests and tools):
 * logits as in dp_score_centroids, sel_ids as in dp_topp_select. */
typedef struct {
  size_t logits, sel_ids, row_start, chunk_entry, counts, partials, total;
  int32_t splits;      /* partial results per head in stage 3          */
  int32_t chunk_rows;  /* granularity (rows) of the stage-3 work split */
  size_t summaries;    /* float2 [heads, ceil(max_clusters_per_seg / 16)]: per head and run of 16 clusters the
                          largest logit and the sum of exp(logit - that), left by the scoring stage */
} dp_workspace_layout;
dp_status dp_get_workspace_layout(const dp_problem *problem, dp_workspace_layout *layout /* host */);

/* Measurement aid (not part of the method): one launch that reads `bytes` bytes of `buffer` (device, 16-byte
 * aligned, bytes a multiple of 16) once, with the access shape of the scoring stage (256 threads per workgroup, four
 * 16-byte loads in flight per thread, 16 KiB of consecutive bytes per workgroup), and writes nothing (sink: a device
 * word that keeps the loads alive, may be NULL).  Its duration is the floor for any single launch that must read
 * that many bytes on this machine.  start_event / stop_event (hipEvent_t as void*, either may be NULL) receive the
 * kernel's own begin and end timestamps, as in dp_score_centroids_timed. */
dp_status dp_stream_read_probe(const void *buffer, size_t bytes, uint32_t *sink, void *stream, void *start_event,
                               void *stop_event);

const char *dp_status_string(dp_status status);

#ifdef __cplusplus
}
#endif
#endif /* DP_H */
