// Host-side launch interface between the C ABI (dp_api.hip) and the kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dp {

constexpr int kHeadDim = 128;  // the only supported head dimension

// rows of one stage-3 work chunk; item boundaries are multiples of it
constexpr int kChunkRows = 64;
// stage 3 pulls (head, split) items from a device-side queue: heads served per launch, workgroups per launch
constexpr int kMaxQueueHeads = 1024;
constexpr int kMaxSplits = 256;  // most partial slots per head
constexpr int kDecodeGrid = 1280;

struct CacheView {
  int32_t batch, n_kv_heads, n_q_heads, group;  // group = n_q_heads / n_kv_heads
  const void *q, *k_cache, *v_cache, *k_centroids, *v_centroids;
  const int64_t *seg_row_base;
  const int32_t *seg_cluster_ptr, *cluster_offsets, *cluster_sizes;
  const uint8_t *cluster_flags;  // nullable
  int32_t max_clusters_per_seg, max_rows_per_seg;
  int32_t uniform_kc;  // > 0 when the host can tell that every segment has exactly this many clusters
  float sm_scale;
};

// Per-head stage-2 -> stage-3 plan, all int32, head-major:
//   ent_src  [nh, max_k]      exact entry: first row of the cluster relative to the segment;
//                             approximated entry: segment-local cluster id
//   row_start[nh, max_k + 1]  exclusive prefix of rows over the entry list
//                             (an exact cluster has s_i rows, an approximated one has 1)
//   chunk_entry[nh, chunk_stride]  entry that holds row q*kChunkRows
//   head_rows[nh]             total rows of the head; -1: the head has already been attended
//   done[nh]                  arrival counter of the head's decode workgroups (zeroed by the planner)
struct Plan {
  int32_t *ent_src, *row_start, *chunk_entry, *head_rows, *done;
  int32_t *queue_next;  // one item counter per slab of kMaxQueueHeads heads (zeroed by the planner)
  // nullable: per slab, how many heads the selection kernel left for the decode kernel.  Zeroed by the scoring
  // kernel of the same step; a decode launch that reads 0 returns at once.
  int32_t *pending;
  int32_t chunk_stride;
};

// where attention results go; out == nullptr: nowhere (selection only)
struct AttnOut {
  void *out;
  float *lse;  // nullable
  int32_t out_is_bf16;
};

struct SelectOut {
  int32_t *sel_ids;  // [nh, max_k]
  int32_t *n_exact, *n_retained, *n_exact_tokens;  // [nh]
  // nullable: second copies of the three counts (the caller's optional outputs of the one-call entry points)
  int32_t *n_exact_copy = nullptr, *n_retained_copy = nullptr, *n_exact_tokens_copy = nullptr;
};

// start / stop (nullable): HIP events that receive the kernel's own begin and end timestamps
// zero_words (nullable): n_zero int32 that the kernel clears (the step's pending counters)
// summaries (nullable): float2 [heads, sub_stride]: per head and sub-tile of kSubTile consecutive clusters of its
// segment, (max logit, sum over the sub-tile of exp(logit - that max)); entries beyond the segment's last
// sub-tile are not written
constexpr int kSubTile = 16;
hipError_t launch_score(const CacheView &c, float *logits, hipStream_t s, hipEvent_t start = nullptr,
                        hipEvent_t stop = nullptr, int32_t *zero_words = nullptr, int n_zero = 0,
                        float2 *summaries = nullptr, int sub_stride = 0);

// How stage 2 cuts the order (logit descending, index ascending):
//   by_count == 0: the two top-p thresholds p1, p2 (p2_absolute: p2 is a mass of the whole distribution)
//   by_count != 0: fixed budget, the first k_retained clusters are retained and the first k_exact of them exact
struct SelectRule {
  float p1, p2;
  uint32_t p2_absolute;
  int32_t by_count, k_retained, k_exact;
};

// plan.ent_src == nullptr => no plan is written
// With a plan and attn.out != nullptr, heads with few rows are attended inside the selection kernel.
// The stage-3 queue inside the selection launch (for launches that serve at most kSameLaunchMaxHeads heads):
// the heads that the selection does not attend itself are split over the same launch's workgroups, so no decode
// launch follows.  planned: one counter; it, plan.pending[0] and plan.queue_next[0] must be zero when the launch
// starts (launch_score's zero_words).
constexpr int kSameLaunchMaxHeads = 128;
struct SameLaunchQueue {
  float *partials;
  int splits;
  int32_t *planned;
};
// summaries (nullable): what launch_score left for these logits; lets peaked heads skip reading their logits
hipError_t launch_select(const CacheView &c, const float *logits, const SelectRule &rule, const SelectOut &out,
                         const Plan &plan, const AttnOut &attn, hipStream_t s, hipEvent_t start = nullptr,
                         hipEvent_t stop = nullptr, const float2 *summaries = nullptr, int sub_stride = 0,
                         const SameLaunchQueue *queue = nullptr);

// builds the plan from caller-given sets
hipError_t launch_plan(const CacheView &c, const int32_t *sel_ids, const int32_t *n_exact,
                       const int32_t *n_retained, int32_t *n_exact_tokens, const Plan &plan, const AttnOut &attn,
                       hipStream_t s);

hipError_t launch_decode(const CacheView &c, const int32_t *n_exact, const int32_t *n_retained, const Plan &plan,
                         float *partials, int splits, const AttnOut &attn, hipStream_t s, hipEvent_t start = nullptr,
                         hipEvent_t stop = nullptr, const void *k_gather = nullptr, const void *v_gather = nullptr,
                         int rows_cap = 0);

// A/B variants in the structure of the paper's own kernels (dp_variants.hip)
constexpr int kSortedSelectMaxClusters = 8192;
hipError_t launch_select_sorted(const CacheView &c, const float *logits, const SelectRule &rule, const SelectOut &out,
                                hipStream_t s);
hipError_t launch_gather_rows(const CacheView &c, const int32_t *n_exact, const Plan &plan, void *k_buf, void *v_buf,
                              int rows_cap, hipStream_t s);

// A/B variant: selection per GQA group (dp_union.hip).  launch_group_union turns the heads' lists into one
// list per segment (exact ids ascending, then approximated ids ascending); launch_group_decode attends every head of
// a group over its segment's list (seg_plan: a Plan built with segments in the place of heads; partials: room for
// nh * splits * (kHeadDim + 2) floats).
constexpr int kGroupUnionMaxClusters = 65536;
hipError_t launch_group_union(const CacheView &c, const int32_t *sel_ids, const int32_t *n_exact,
                              const int32_t *n_retained, int32_t *union_ids, int32_t *n_exact_u,
                              int32_t *n_retained_u, hipStream_t s);
hipError_t launch_group_decode(const CacheView &c, const int32_t *n_exact_u, const int32_t *n_retained_u,
                               const Plan &seg_plan, float *partials, int splits, const AttnOut &attn, hipStream_t s);

// Dense attention over rows [seg_row_base[seg], + seg_rows[seg]) of every segment for all its query heads.
// partials: room for nh * max_splits * (kHeadDim + 2) floats.
hipError_t launch_dense(const CacheView &c, const int32_t *seg_rows, float *partials, int max_splits,
                        const AttnOut &attn, hipStream_t s);

// Prefill side: token-order K / V + cluster ids -> cluster-contiguous cache and cluster metadata.
struct BuildProblem {
  int32_t n_seg;
  const void *k_tokens, *v_tokens;
  const int32_t *assignment;
  const int64_t *seg_row_base;
  const int32_t *seg_rows, *seg_cluster_ptr;
  int32_t max_kc, max_rows;
  void *k_cache, *v_cache, *k_centroids, *v_centroids;
  int32_t *cluster_offsets, *cluster_sizes, *token_row;  // token_row nullable
  float *v_sums;                                         // nullable
};
void build_workspace_layout(int n_seg, int max_rows, int max_kc, size_t *hist_bytes, size_t *rank_bytes,
                            size_t *row_token_bytes, int *n_blocks);
hipError_t launch_build(const BuildProblem &p, void *workspace, hipStream_t s);

// k-means assignment step: nearest centroid of every token (dp_kmeans.hip)
struct KmeansProblem {
  int32_t n_seg;
  const void *k_tokens, *centroids;
  const int64_t *seg_row_base;
  const int32_t *seg_rows, *seg_cluster_ptr;
  int32_t max_rows, total_clusters;
  int32_t *assignment;
  float *best_score;  // nullable
};
hipError_t launch_kmeans_assign(const KmeansProblem &p, float *half_norm, hipStream_t s);
// centroids[c] of a segment with n tokens and kc clusters = the key of token floor(c * n / kc) (zero if n == 0)
hipError_t launch_kmeans_init_strided(const KmeansProblem &p, void *centroids, int max_kc, hipStream_t s);

// largest max_clusters_per_seg the selection kernel supports
constexpr int kSelectMaxClusters = 65536;

}  // namespace dp
