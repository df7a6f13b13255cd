/*
 * Double-P decode attention: plain fp64 CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, obviously-correct statement of
 * what one decode step of hierarchical top-p sparse attention computes, written
 * from the paper's equations (Sec. 2.1 Eq. 1; Sec. 4.1 Eq. 2; Sec. 4.2 Eq. 3-7;
 * Sec. 4.3 Eq. 8-9).  It shares no code with the HIP library, is never called
 * by it, and is used only by the tests, the smoke check and the bench's
 * reported CPU baseline.
 *
 * All arithmetic is IEEE double.  Stored tensors are bf16 bit patterns
 * (uint16_t) that are widened exactly.  Every pointer is a HOST pointer owned
 * by the caller; nothing is retained between calls.
 *
 * Pins (tests, CPU only): dense limit p1 = p2 = 1 against an independent
 * scipy softmax; singleton clusters; zero-variance clusters (output
 * independent of p2); Jensen bound on the estimated cluster mass; p2 = 0
 * closed form; mass >= p and minimality; brute-force subset enumeration on
 * tiny inputs; permutation and size-scaling invariances.
 * Parity unpinned: which distribution the second top-p runs on (the paper
 * gives no equation and prints no value that separates the two readings kept
 * here, see DPO_P2_ABSOLUTE).
 */
#ifndef DP_ORACLE_H
#define DP_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int32_t batch, n_kv_heads, n_q_heads, head_dim;
  const uint16_t *q;              /* bf16 [batch, n_q_heads, head_dim]                       */
  const uint16_t *k_cache;        /* bf16 [total_rows, head_dim], cluster-contiguous         */
  const uint16_t *v_cache;        /* bf16 [total_rows, head_dim], same row order             */
  const int64_t *seg_row_base;    /* [batch*n_kv_heads] first cache row of segment b*Hkv+g   */
  const int32_t *seg_cluster_ptr; /* [batch*n_kv_heads+1] CSR into the per-cluster arrays    */
  const int32_t *cluster_offsets; /* [total_clusters] first row, relative to seg_row_base    */
  const int32_t *cluster_sizes;   /* [total_clusters] s_i >= 0; 0 = empty, never selected    */
  const uint16_t *k_centroids;    /* bf16 [total_clusters, head_dim]  C_i                    */
  const uint16_t *v_centroids;    /* bf16 [total_clusters, head_dim]  mean value of cluster  */
  double sm_scale;                /* 0 => 1/sqrt(head_dim)                                   */
  const uint8_t *cluster_flags;   /* [total_clusters] DPO_CLUSTER_* bits; NULL = none set     */
} dpo_cache;

/* A pinned cluster holds tokens that every method keeps dense (the sink and
 * sliding-window tokens of Sec. 5.1): it takes no part in the cluster
 * distribution (Eq. 6, Eq. 7 and the second top-p run over the other, "middle"
 * clusters only) and its tokens are always in the exact token set of Eq. 8/9. */
#define DPO_CLUSTER_PINNED 1u

/* Second top-p reading: default = threshold p2 * (mass retained by the first
 * top-p); with this flag = min(p2, that mass), i.e. p2 on the full distribution. */
#define DPO_P2_ABSOLUTE 1u

/* number of clusters of the KV segment that query head h of sequence b reads */
int32_t dpo_num_clusters(const dpo_cache *c, int32_t b, int32_t h);

/* Eq. 3 + Eq. 5: logit[i] = q.C_i/sqrt(d) + ln s_i  (= log Zhat_i); -inf if s_i == 0. */
void dpo_centroid_logits(const dpo_cache *c, int32_t b, int32_t h, double *logit);

/* dpo_centroid_logits with the pinned clusters set to -inf: the logits of the
 * candidates of the cluster distribution. */
void dpo_candidate_logits(const dpo_cache *c, int32_t b, int32_t h, double *logit);

/* Pinned, non-empty clusters of the head's segment in ascending order; returns
 * their number. ids: room for dpo_num_clusters entries. */
int32_t dpo_pinned_clusters(const dpo_cache *c, int32_t b, int32_t h, int32_t *ids);

/* Eq. 6: A_hat = softmax(logit) over the n clusters (empty clusters get 0). */
void dpo_cluster_distribution(const double *logit, int32_t n, double *a_hat);

/* Order used by Eq. 7: non-empty clusters by logit descending, ties by index
 * ascending. Writes the permutation to order[0..ret) and returns ret. */
int32_t dpo_sorted_order(const double *logit, int32_t n, int32_t *order);

/* Eq. 7 and the second top-p (Sec. 4.3). cum[k] (k < n_nonempty) receives the
 * mass of the first k+1 clusters of the order. Returns k1 and k2 (clusters
 * order[0..k2) are exact, order[k2..k1) are approximated) and m1 = cum[k1-1]. */
void dpo_double_top_p(const double *a_hat, const int32_t *order, int32_t n_nonempty, double p1, double p2,
                      uint32_t flags, double *cum, int32_t *k1, int32_t *k2, double *m1);

/* Eq. 8 + Eq. 9 for the given sets (segment-local cluster ids). out[d] and
 * lse = ln Z~ ; with both sets empty out = 0 and lse = -inf. */
void dpo_mixed_attention(const dpo_cache *c, int32_t b, int32_t h, const int32_t *exact_ids, int32_t n_exact,
                         const int32_t *approx_ids, int32_t n_approx, double *out, double *lse);

/* Eq. 1 over every token of the head's segment. */
void dpo_dense_attention(const dpo_cache *c, int32_t b, int32_t h, double *out, double *lse);

/* Eq. 4: log_z[i] = ln sum_j exp(x_ij) per cluster (-inf if empty). */
void dpo_exact_cluster_log_mass(const dpo_cache *c, int32_t b, int32_t h, double *log_z);

/* The whole decode step for every (b, h): stages in the order above, on the
 * candidate logits; the exact set is order[0..k2) plus the pinned clusters.
 * out [batch*n_q_heads*d], lse/k1/k2 [batch*n_q_heads]; order (nullable)
 * [batch*n_q_heads, order_stride] receives each head's sorted order.
 * n_threads <= 1 runs serially, else OpenMP over (b, h). Returns the number of
 * threads used. */
int32_t dpo_decode_step(const dpo_cache *c, double p1, double p2, uint32_t flags, double *out, double *lse,
                        int32_t *k1, int32_t *k2, int32_t *order, int64_t order_stride, int32_t n_threads);

/* Fixed budget in place of the two thresholds (the fixed top-k cluster retrieval of
 * the cluster-based baseline, Sec. 5.1): of the n_nonempty clusters of the order
 * the first k1 = min(max(k_retained, 0), n_nonempty) are retained and the first
 * k2 = min(max(k_exact, 0), k1) of them are exact. */
void dpo_fixed_budget(int32_t n_nonempty, int32_t k_retained, int32_t k_exact, int32_t *k1, int32_t *k2);

/* The decode step with dpo_fixed_budget in place of dpo_double_top_p; same
 * outputs and threading as dpo_decode_step. */
int32_t dpo_budget_step(const dpo_cache *c, int32_t k_retained, int32_t k_exact, double *out, double *lse,
                        int32_t *k1, int32_t *k2, int32_t *order, int64_t order_stride, int32_t n_threads);

/* Eq. 1 for every (b, h), same threading. */
int32_t dpo_dense_step(const dpo_cache *c, double *out, double *lse, int32_t n_threads);

/* Prefill side (Sec. 4.1, Eq. 2): from K / V in token order and each token's
 * cluster id, the cluster-contiguous cache and the per-cluster metadata that the
 * decode step reads.  Segment seg owns rows [seg_row_base[seg], + seg_rows[seg])
 * of the token arrays and of the output cache, and clusters [ptr[seg], ptr[seg+1]).
 * Clusters are laid out in index order, the tokens of a cluster in token order.
 *   cluster_sizes s_i, cluster_offsets (exclusive prefix of the sizes),
 *   k_centroids C_i = mean key, v_centroids = V^Sigma_i / s_i, both rounded once
 *   to bf16 (ties to even; zero rows for an empty cluster), v_sums (nullable)
 *   V^Sigma_i in double, token_row (nullable) the segment-relative cache row of each token.
 * A token whose id is outside [0, clusters of the segment) is left out (token_row -1). */
void dpo_build_cluster_cache(int32_t n_seg, int32_t d, const uint16_t *k_tokens, const uint16_t *v_tokens,
                             const int32_t *assignment, const int64_t *seg_row_base, const int32_t *seg_rows,
                             const int32_t *seg_cluster_ptr, uint16_t *k_cache, uint16_t *v_cache,
                             int32_t *cluster_offsets, int32_t *cluster_sizes, uint16_t *k_centroids,
                             uint16_t *v_centroids, double *v_sums, int32_t *token_row);

/* Assignment step of the k-means clustering of the keys (Sec. 4.1): every token
 * goes to the nearest centroid of its segment (Euclidean distance), the lower
 * index on a tie; written as argmax of x.c - |c|^2 / 2, which differs from
 * -|x - c|^2 / 2 by a constant per token.  best_score / runner_up (nullable):
 * the largest and the second largest of those scores (-inf if there is none). */
void dpo_kmeans_assign(int32_t n_seg, int32_t d, const uint16_t *k_tokens, const uint16_t *centroids,
                       const int64_t *seg_row_base, const int32_t *seg_rows, const int32_t *seg_cluster_ptr,
                       int32_t *assignment, double *best_score, double *runner_up);

#ifdef __cplusplus
}
#endif
#endif
