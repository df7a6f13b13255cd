// C ABI of the Double-P decode-attention library (see include/dp.h): argument
// checks, workspace layout and kernel sequencing.  No allocation, no
// synchronisation, no state.
#include "dp.h"

#include <math.h>

#include <atomic>

#include "dp_kernels.hpp"

namespace {

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

bool shape_ok(const dp_problem *p) {
  return p && p->batch > 0 && p->n_kv_heads > 0 && p->n_q_heads > 0 && p->n_q_heads % p->n_kv_heads == 0 &&
         p->total_clusters >= 0 && p->max_clusters_per_seg >= 0 && p->max_rows_per_seg >= 0 &&
         p->max_clusters_per_seg <= p->total_clusters && !(p->sm_scale < 0.0f) && p->sm_scale == p->sm_scale;
}

dp_status supported(const dp_problem *p) {
  if (p->head_dim != dp::kHeadDim) return DP_ERR_UNSUPPORTED;
  if (p->n_q_heads / p->n_kv_heads > 16) return DP_ERR_UNSUPPORTED;  // one DPP-row lane per head of the group
  if (p->max_clusters_per_seg > dp::kSelectMaxClusters) return DP_ERR_UNSUPPORTED;
  return DP_OK;
}

bool pointers_ok(const dp_problem *p) {
  return p->q && p->seg_row_base && p->seg_cluster_ptr &&
         (p->total_clusters == 0 ||
          (p->cluster_offsets && p->cluster_sizes && p->k_centroids && p->v_centroids && p->k_cache && p->v_cache));
}

dp::CacheView view_of(const dp_problem *p) {
  dp::CacheView c;
  c.batch = p->batch;
  c.n_kv_heads = p->n_kv_heads;
  c.n_q_heads = p->n_q_heads;
  c.group = p->n_q_heads / p->n_kv_heads;
  c.q = p->q;
  c.k_cache = p->k_cache;
  c.v_cache = p->v_cache;
  c.k_centroids = p->k_centroids;
  c.v_centroids = p->v_centroids;
  c.seg_row_base = p->seg_row_base;
  c.seg_cluster_ptr = p->seg_cluster_ptr;
  c.cluster_offsets = p->cluster_offsets;
  c.cluster_sizes = p->cluster_sizes;
  c.cluster_flags = p->cluster_flags;
  c.max_clusters_per_seg = p->max_clusters_per_seg;
  c.max_rows_per_seg = p->max_rows_per_seg;
  // every segment holds <= max clusters and they sum to total: equality means all are full
  const int64_t n_seg = (int64_t)p->batch * p->n_kv_heads;
  c.uniform_kc = (p->max_clusters_per_seg > 0 && n_seg * p->max_clusters_per_seg == p->total_clusters)
                     ? p->max_clusters_per_seg
                     : 0;
  c.sm_scale = p->sm_scale != 0.0f ? p->sm_scale : 1.0f / sqrtf((float)p->head_dim);
  return c;
}

// stage-3 splits per head: aim at several thousand workgroups in total, many more than the 256 CUs can
// hold at once, so that the last round of workgroups is short against the whole
constexpr long kSplitTarget = 16384;
int choose_splits(const dp_problem *p) {
  const long nh = (long)p->batch * p->n_q_heads;
  long s = (kSplitTarget + nh - 1) / nh;
  const long by_rows = ((long)p->max_rows_per_seg + p->max_clusters_per_seg + dp::kChunkRows - 1) / dp::kChunkRows;
  if (s > by_rows) s = by_rows;
  if (s > dp::kMaxSplits) s = dp::kMaxSplits;
  if (s < 8) s = 8;
  if (s > by_rows && by_rows >= 1) s = by_rows;
  if (s < 1) s = 1;
  return (int)s;
}

void layout_of(const dp_problem *p, dp_workspace_layout *L) {
  const size_t nh = (size_t)p->batch * p->n_q_heads;
  const size_t mk = (size_t)p->max_clusters_per_seg;
  const size_t chunk_stride = ((size_t)p->max_rows_per_seg + mk) / dp::kChunkRows + 2;
  const int splits = choose_splits(p);
  size_t off = 0;
  L->logits = off;
  off = align_up(off + sizeof(float) * (size_t)(p->n_q_heads / p->n_kv_heads) * (size_t)p->total_clusters, 256);
  L->sel_ids = off;
  off = align_up(off + sizeof(int32_t) * nh * mk, 256);
  size_t ent_src = off;  // plan.ent_src shares the layout slot directly after sel_ids
  off = align_up(off + sizeof(int32_t) * nh * mk, 256);
  L->row_start = off;
  off = align_up(off + sizeof(int32_t) * nh * (mk + 1), 256);
  L->chunk_entry = off;
  off = align_up(off + sizeof(int32_t) * nh * chunk_stride, 256);
  // n_exact, n_retained, n_exact_tokens, done, head_rows : 5 x [nh]; then per slab of heads the queue and the pending
  // counter, then the count of heads whose selection is complete (head_rows .. that count: one run of words, so the
  // scoring kernel can clear them together)
  L->counts = off;
  off = align_up(off + sizeof(int32_t) * (5 * nh + 2 * ((nh + dp::kMaxQueueHeads - 1) / dp::kMaxQueueHeads) + 1), 256);
  L->partials = off;
  off = align_up(off + sizeof(float) * nh * (size_t)splits * (dp::kHeadDim + 2), 256);
  L->summaries = off;  // (max, sum exp) per head and sub-tile of kSubTile clusters
  off = align_up(off + sizeof(float2) * nh * ((mk + dp::kSubTile - 1) / dp::kSubTile), 256);
  L->total = off;
  L->splits = splits;
  L->chunk_rows = dp::kChunkRows;
  (void)ent_src;
}

struct Workspace {
  float *logits;
  int32_t *sel_ids, *n_exact, *n_retained, *n_exact_tokens;
  dp::Plan plan;
  int32_t *planned;
  float *partials;
  float2 *summaries;
  int sub_stride;
  int splits;
};

Workspace carve(const dp_problem *p, void *ws) {
  dp_workspace_layout L;
  layout_of(p, &L);
  char *b = static_cast<char *>(ws);
  const size_t nh = (size_t)p->batch * p->n_q_heads;
  const size_t mk = (size_t)p->max_clusters_per_seg;
  Workspace w;
  w.logits = reinterpret_cast<float *>(b + L.logits);
  w.sel_ids = reinterpret_cast<int32_t *>(b + L.sel_ids);
  w.plan.ent_src = reinterpret_cast<int32_t *>(b + align_up(L.sel_ids + sizeof(int32_t) * nh * mk, 256));
  w.plan.row_start = reinterpret_cast<int32_t *>(b + L.row_start);
  w.plan.chunk_entry = reinterpret_cast<int32_t *>(b + L.chunk_entry);
  w.plan.chunk_stride = (int32_t)(((size_t)p->max_rows_per_seg + mk) / dp::kChunkRows + 2);
  int32_t *counts = reinterpret_cast<int32_t *>(b + L.counts);
  w.n_exact = counts;
  w.n_retained = counts + nh;
  w.n_exact_tokens = counts + 2 * nh;
  w.plan.done = counts + 3 * nh;
  w.plan.head_rows = counts + 4 * nh;
  w.plan.queue_next = counts + 5 * nh;
  w.plan.pending = nullptr;  // the one-call path turns it on (its scoring kernel clears the counters)
  w.planned = w.plan.queue_next + 2 * ((nh + dp::kMaxQueueHeads - 1) / dp::kMaxQueueHeads);
  w.partials = reinterpret_cast<float *>(b + L.partials);
  w.summaries = reinterpret_cast<float2 *>(b + L.summaries);
  w.sub_stride = (int)((mk + dp::kSubTile - 1) / dp::kSubTile);
  w.splits = L.splits;
  return w;
}

dp_status check_common(const dp_problem *p) {
  if (!shape_ok(p)) return DP_ERR_INVALID_ARG;
  const dp_status s = supported(p);
  if (s != DP_OK) return s;
  if (!pointers_ok(p)) return DP_ERR_INVALID_ARG;
  return DP_OK;
}

bool p_in_domain(float p1, float p2) { return p1 > 0.0f && p1 <= 1.0f && p2 >= 0.0f && p2 <= 1.0f; }

dp::SelectRule top_p_rule(const dp_problem *p, float p1, float p2) {
  return dp::SelectRule{p1, p2, p->flags & DP_FLAG_P2_ABSOLUTE, 0, 0, 0};
}
dp::SelectRule budget_rule(int32_t k_retained, int32_t k_exact) {
  return dp::SelectRule{1.0f, 1.0f, 0u, 1, k_retained, k_exact};
}

dp_status select_only(const dp_problem *problem, const float *logits, const dp::SelectRule &rule, int32_t *sel_ids,
                      int32_t *n_exact, int32_t *n_retained, int32_t *n_exact_tokens, void *stream) {
  if (!n_exact || !n_retained || !n_exact_tokens) return DP_ERR_INVALID_ARG;
  if (problem->max_clusters_per_seg > 0 && (!logits || !sel_ids)) return DP_ERR_INVALID_ARG;
  dp::SelectOut out{sel_ids, n_exact, n_retained, n_exact_tokens};
  dp::Plan none{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0};
  dp::AttnOut nowhere{nullptr, nullptr, 0};
  return dp::launch_select(view_of(problem), logits, rule, out, none, nowhere, static_cast<hipStream_t>(stream)) ==
                 hipSuccess
             ? DP_OK
             : DP_ERR_HIP;
}

// Whether a step runs the split decode inside the selection launch.
// Where the shared launch pays (measured, 32 heads, us per step against three launches): it saves the decode launch
// of a step whose heads are all attended inline (8192 clusters per KV head: 13.3 against 14.7; 2048 clusters: 12.0
// against 14.9), and it starts the queue without a launch in between when only some heads are flat (one flat head
// in eight: 30.3 against 31.8 at 2048 clusters, 50.5 against 55.9 at 8192).  A step of flat heads only is served
// more slowly by the selection kernel's few large workgroups than by the decode kernel's many small ones (2048
// clusters: 46 against 43; 8192: 93 against 84): the flag below is for a caller who knows.  With more heads than
// kSameLaunchMaxHeads the selecting workgroups come in rounds and the shared launch loses (512 peaked heads: 29.6
// against 24.3).  Top-p rule only (a fixed budget leaves rows on every head).
bool shares_launch(const dp_problem *problem, bool by_count) {
  const int mk = problem->max_clusters_per_seg;
  const int64_t nh = (int64_t)problem->batch * problem->n_q_heads;
  // (the scoring kernel clears 256 words per segment for the step: the shared launch needs one per head and three more)
  return mk > 0 && nh <= dp::kSameLaunchMaxHeads && nh + 3 <= 256 * (int64_t)problem->batch * problem->n_kv_heads &&
         !by_count && !(problem->flags & DP_FLAG_SEPARATE_DECODE_LAUNCH);
}

// score -> select (+ attention of light heads) -> split decode, on one stream.  A step that serves few heads runs
// the split decode inside the selection launch (two launches); flags bit DP_FLAG_SEPARATE_DECODE_LAUNCH keeps the
// three launches.
dp_status whole_step(const dp_problem *problem, const dp::SelectRule &rule, void *out, dp_dtype out_dtype, float *lse,
                     int32_t *n_exact, int32_t *n_retained, int32_t *n_exact_tokens, void *workspace,
                     size_t workspace_bytes, void *stream, void *const *events = nullptr) {
  hipEvent_t ev[6] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
  if (events)
    for (int i = 0; i < 6; ++i) ev[i] = static_cast<hipEvent_t>(events[i]);
  if (out_dtype != DP_BF16 && out_dtype != DP_F32) return DP_ERR_UNSUPPORTED;
  if (!out || !workspace) return DP_ERR_INVALID_ARG;
  if (workspace_bytes < dp_workspace_bytes(problem)) return DP_ERR_WORKSPACE_TOO_SMALL;
  if (reinterpret_cast<uintptr_t>(workspace) % 256) return DP_ERR_INVALID_ARG;
  const dp::CacheView c = view_of(problem);
  Workspace w = carve(problem, workspace);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int n_slabs = (int)(((size_t)problem->batch * problem->n_q_heads + dp::kMaxQueueHeads - 1) / dp::kMaxQueueHeads);
  if (problem->max_clusters_per_seg > 0 && n_slabs <= 64) w.plan.pending = w.plan.queue_next + n_slabs;
  const int nh_i = problem->batch * problem->n_q_heads;
  const bool same_launch = w.plan.pending && shares_launch(problem, rule.by_count != 0);
  // the summaries serve the top-p rule on heads without cluster flags
  float2 *summ = (!rule.by_count && !problem->cluster_flags && rule.p1 < 1.0f) ? w.summaries : nullptr;
  // the scoring kernel clears the step's counters: item counters, pending counters, planned (contiguous), and
  // in front of them head_rows when the queue runs inside the selection launch (only heads with rows write it then)
  int32_t *zero = !w.plan.pending ? nullptr : same_launch ? w.plan.head_rows : w.plan.queue_next;
  const int n_zero = 2 * n_slabs + 1 + (same_launch ? nh_i : 0);
  if (dp::launch_score(c, w.logits, s, ev[0], ev[1], zero, n_zero, summ, w.sub_stride) != hipSuccess) return DP_ERR_HIP;
  // the optional count outputs are written by the selection kernel next to the workspace's own
  dp::SelectOut so{w.sel_ids, w.n_exact, w.n_retained, w.n_exact_tokens, n_exact, n_retained, n_exact_tokens};
  const dp::AttnOut attn{out, lse, out_dtype == DP_BF16};
  if (same_launch) {
    const dp::SameLaunchQueue q{w.partials, w.splits, w.planned};
    if (dp::launch_select(c, w.logits, rule, so, w.plan, attn, s, ev[2], ev[3], summ, w.sub_stride, &q) != hipSuccess)
      return DP_ERR_HIP;
    // measurement: there is no decode launch; its two events mark the end of the step
    if (ev[4] && hipEventRecord(ev[4], s) != hipSuccess) return DP_ERR_HIP;
    if (ev[5] && hipEventRecord(ev[5], s) != hipSuccess) return DP_ERR_HIP;
    return DP_OK;
  }
  if (dp::launch_select(c, w.logits, rule, so, w.plan, attn, s, ev[2], ev[3], summ, w.sub_stride) != hipSuccess)
    return DP_ERR_HIP;
  if (dp::launch_decode(c, w.n_exact, w.n_retained, w.plan, w.partials, w.splits, attn, s, ev[4], ev[5]) !=
      hipSuccess)
    return DP_ERR_HIP;
  return DP_OK;
}

// ---- workspace of dp_decode_attention_static: a device array that lives in the library's code object ----
// Every GPU that loads the library holds its own copy until the process ends.  In host code the array's name
// only stands for the symbol; its device address on the current device comes from hipGetSymbolAddress, once per
// device, and only that pointer is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[DP_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];  // per device: the address of `scratch` there, nullptr until asked

dp_status static_scratch(void **ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return DP_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return DP_ERR_UNSUPPORTED;
  void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    // first call on this device (it is the current one); threads that race here get the same address
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DP_ERR_HIP;
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *ptr = p;
  return DP_OK;
}

}  // namespace

extern "C" {

size_t dp_workspace_bytes(const dp_problem *problem) {
  if (!shape_ok(problem)) return 0;
  dp_workspace_layout L;
  layout_of(problem, &L);
  return L.total;
}

size_t dp_logits_count(const dp_problem *problem) {
  if (!shape_ok(problem)) return 0;
  return (size_t)(problem->n_q_heads / problem->n_kv_heads) * (size_t)problem->total_clusters;
}

dp_status dp_get_workspace_layout(const dp_problem *problem, dp_workspace_layout *layout) {
  if (!shape_ok(problem) || !layout) return DP_ERR_INVALID_ARG;
  layout_of(problem, layout);
  return DP_OK;
}

dp_status dp_score_centroids(const dp_problem *problem, float *logits, void *stream) {
  dp_status st = check_common(problem);
  if (st != DP_OK) return st;
  if (!logits && problem->total_clusters > 0) return DP_ERR_INVALID_ARG;
  if (problem->total_clusters == 0) return DP_OK;
  return dp::launch_score(view_of(problem), logits, static_cast<hipStream_t>(stream)) == hipSuccess ? DP_OK
                                                                                                   : DP_ERR_HIP;
}

dp_status dp_score_centroids_timed(const dp_problem *problem, float *logits, void *stream, void *start_event,
                                   void *stop_event) {
  dp_status st = check_common(problem);
  if (st != DP_OK) return st;
  if (!logits && problem->total_clusters > 0) return DP_ERR_INVALID_ARG;
  if (problem->total_clusters == 0) return DP_OK;
  return dp::launch_score(view_of(problem), logits, static_cast<hipStream_t>(stream),
                          static_cast<hipEvent_t>(start_event), static_cast<hipEvent_t>(stop_event)) == hipSuccess
             ? DP_OK
             : DP_ERR_HIP;
}

dp_status dp_topp_select(const dp_problem *problem, const float *logits, float p1, float p2, int32_t *sel_ids,
                         int32_t *n_exact, int32_t *n_retained, int32_t *n_exact_tokens, void *stream) {
  dp_status st = check_common(problem);
  if (st != DP_OK) return st;
  if (!p_in_domain(p1, p2)) return DP_ERR_INVALID_ARG;
  return select_only(problem, logits, top_p_rule(problem, p1, p2), sel_ids, n_exact, n_retained, n_exact_tokens,
                     stream);
}

dp_status dp_topp_select_sorted(const dp_problem *problem, const float *logits, float p1, float p2, int32_t *sel_ids,
                                int32_t *n_exact, int32_t *n_retained, int32_t *n_exact_tokens, void *stream) {
  dp_status st = check_common(problem);
  if (st != DP_OK) return st;
  if (!p_in_domain(p1, p2)) return DP_ERR_INVALID_ARG;
  if (problem->max_clusters_per_seg > dp::kSortedSelectMaxClusters || problem->cluster_flags) return DP_ERR_UNSUPPORTED;
  if (!n_exact || !n_retained || !n_exact_tokens) return DP_ERR_INVALID_ARG;
  if (problem->max_clusters_per_seg > 0 && (!logits || !sel_ids)) return DP_ERR_INVALID_ARG;
  dp::SelectOut out{sel_ids, n_exact, n_retained, n_exact_tokens};
  return dp::launch_select_sorted(view_of(problem), logits, top_p_rule(problem, p1, p2), out,
                                  static_cast<hipStream_t>(stream)) == hipSuccess
             ? DP_OK
             : DP_ERR_HIP;
}

dp_status dp_topk_select(const dp_problem *problem, const float *logits, int32_t k_retained, int32_t k_exact,
                         int32_t *sel_ids, int32_t *n_exact, int32_t *n_retained, int32_t *n_exact_tokens,
                         void *stream) {
  dp_status st = check_common(problem);
  if (st != DP_OK) return st;
  if (k_retained < 0 || k_exact < 0) return DP_ERR_INVALID_ARG;
  return select_only(problem, logits, budget_rule(k_retained, k_exact), sel_ids, n_exact, n_retained, n_exact_tokens,
                     stream);
}

dp_status dp_sparse_decode(const dp_problem *problem, const int32_t *sel_ids, const int32_t *n_exact,
                           const int32_t *n_retained, const int32_t *n_exact_tokens, void *out, dp_dtype out_dtype,
                           float *lse, void *workspace, size_t workspace_bytes, void *stream) {
  (void)n_exact_tokens;
  dp_status st = check_common(problem);
  if (st != DP_OK) return st;
  if (out_dtype != DP_BF16 && out_dtype != DP_F32) return DP_ERR_UNSUPPORTED;
  if (!n_exact || !n_retained || !out || !workspace) return DP_ERR_INVALID_ARG;
  if (problem->max_clusters_per_seg > 0 && !sel_ids) return DP_ERR_INVALID_ARG;
  if (workspace_bytes < dp_workspace_bytes(problem)) return DP_ERR_WORKSPACE_TOO_SMALL;
  if (reinterpret_cast<uintptr_t>(workspace) % 256) return DP_ERR_INVALID_ARG;
  const dp::CacheView c = view_of(problem);
  const Workspace w = carve(problem, workspace);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const dp::AttnOut attn{out, lse, out_dtype == DP_BF16};
  if (dp::launch_plan(c, sel_ids, n_exact, n_retained, nullptr, w.plan, attn, s) != hipSuccess) return DP_ERR_HIP;
  if (dp::launch_decode(c, n_exact, n_retained, w.plan, w.partials, w.splits, attn, s) != hipSuccess)
    return DP_ERR_HIP;
  return DP_OK;
}

dp_status dp_sparse_decode_gathered(const dp_problem *problem, const int32_t *sel_ids, const int32_t *n_exact,
                                    const int32_t *n_retained, void *out, dp_dtype out_dtype, float *lse,
                                    void *k_buf, void *v_buf, int32_t rows_cap, void *workspace,
                                    size_t workspace_bytes, void *stream) {
  dp_status st = check_common(problem);
  if (st != DP_OK) return st;
  if (out_dtype != DP_BF16 && out_dtype != DP_F32) return DP_ERR_UNSUPPORTED;
  if (!n_exact || !n_retained || !out || !workspace || !k_buf || !v_buf || rows_cap <= 0) return DP_ERR_INVALID_ARG;
  if (problem->max_clusters_per_seg > 0 && !sel_ids) return DP_ERR_INVALID_ARG;
  if (workspace_bytes < dp_workspace_bytes(problem)) return DP_ERR_WORKSPACE_TOO_SMALL;
  if (reinterpret_cast<uintptr_t>(workspace) % 256) return DP_ERR_INVALID_ARG;
  const dp::CacheView c = view_of(problem);
  const Workspace w = carve(problem, workspace);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const dp::AttnOut attn{out, lse, out_dtype == DP_BF16};
  if (dp::launch_plan(c, sel_ids, n_exact, n_retained, nullptr, w.plan, attn, s) != hipSuccess) return DP_ERR_HIP;
  if (dp::launch_gather_rows(c, n_exact, w.plan, k_buf, v_buf, rows_cap, s) != hipSuccess) return DP_ERR_HIP;
  if (dp::launch_decode(c, n_exact, n_retained, w.plan, w.partials, w.splits, attn, s, nullptr, nullptr, k_buf, v_buf,
                        rows_cap) != hipSuccess)
    return DP_ERR_HIP;
  return DP_OK;
}

dp_status dp_group_union_decode_attention(const dp_problem *problem, float p1, float p2, void *out,
                                          dp_dtype out_dtype, float *lse, int32_t *union_ids, int32_t *n_exact_u,
                                          int32_t *n_retained_u, void *workspace, size_t workspace_bytes,
                                          void *stream) {
  dp_status st = check_common(problem);
  if (st != DP_OK) return st;
  if (!p_in_domain(p1, p2)) return DP_ERR_INVALID_ARG;
  if (out_dtype != DP_BF16 && out_dtype != DP_F32) return DP_ERR_UNSUPPORTED;
  if (problem->max_clusters_per_seg > dp::kGroupUnionMaxClusters) return DP_ERR_UNSUPPORTED;
  if (!out || !workspace || !n_exact_u || !n_retained_u) return DP_ERR_INVALID_ARG;
  if (problem->max_clusters_per_seg > 0 && !union_ids) return DP_ERR_INVALID_ARG;
  if (workspace_bytes < dp_workspace_bytes(problem)) return DP_ERR_WORKSPACE_TOO_SMALL;
  if (reinterpret_cast<uintptr_t>(workspace) % 256) return DP_ERR_INVALID_ARG;
  const dp::CacheView c = view_of(problem);
  const Workspace w = carve(problem, workspace);
  hipStream_t s = static_cast<hipStream_t>(stream);
  // per-head sets as in dp_topp_select, into the workspace
  if (dp::launch_score(c, w.logits, s) != hipSuccess) return DP_ERR_HIP;
  const dp::SelectOut per_head{w.sel_ids, w.n_exact, w.n_retained, w.n_exact_tokens};
  const dp::Plan none{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0};
  const dp::AttnOut nowhere{nullptr, nullptr, 0};
  if (dp::launch_select(c, w.logits, top_p_rule(problem, p1, p2), per_head, none, nowhere, s) != hipSuccess)
    return DP_ERR_HIP;
  if (dp::launch_group_union(c, w.sel_ids, w.n_exact, w.n_retained, union_ids, n_exact_u, n_retained_u, s) != hipSuccess)
    return DP_ERR_HIP;
  // the stage-3 plan of the union lists: the planner sees one "head" per segment
  dp::CacheView per_seg = c;
  per_seg.n_q_heads = c.n_kv_heads;
  per_seg.group = 1;
  if (dp::launch_plan(per_seg, union_ids, n_exact_u, n_retained_u, nullptr, w.plan, nowhere, s) != hipSuccess)
    return DP_ERR_HIP;
  const dp::AttnOut attn{out, lse, out_dtype == DP_BF16};
  const int splits = w.splits < 64 ? w.splits : 64;
  if (dp::launch_group_decode(c, n_exact_u, n_retained_u, w.plan, w.partials, splits, attn, s) != hipSuccess)
    return DP_ERR_HIP;
  return DP_OK;
}

dp_status dp_decode_attention(const dp_problem *problem, float p1, float p2, void *out, dp_dtype out_dtype,
                              float *lse, int32_t *n_exact, int32_t *n_retained, int32_t *n_exact_tokens,
                              void *workspace, size_t workspace_bytes, void *stream) {
  dp_status st = check_common(problem);
  if (st != DP_OK) return st;
  if (!p_in_domain(p1, p2)) return DP_ERR_INVALID_ARG;
  return whole_step(problem, top_p_rule(problem, p1, p2), out, out_dtype, lse, n_exact, n_retained, n_exact_tokens,
                    workspace, workspace_bytes, stream);
}

int32_t dp_decode_attention_launches(const dp_problem *problem) {
  if (check_common(problem) != DP_OK) return 0;
  if (problem->max_clusters_per_seg == 0) return 0;
  const int64_t nh = (int64_t)problem->batch * problem->n_q_heads;
  const int score = problem->n_q_heads / problem->n_kv_heads == 3 ? 2 : 1;  // a group of 3 is scored as 2 + 1 heads
  if (shares_launch(problem, false)) return score + 1;
  return score + 1 + (int32_t)((nh + dp::kMaxQueueHeads - 1) / dp::kMaxQueueHeads);
}

dp_status dp_decode_attention_static(const dp_problem *problem, float p1, float p2, void *out, dp_dtype out_dtype,
                                     float *lse, int32_t *n_exact, int32_t *n_retained, int32_t *n_exact_tokens,
                                     void *stream) {
  dp_status st = check_common(problem);
  if (st != DP_OK) return st;
  if (!p_in_domain(p1, p2)) return DP_ERR_INVALID_ARG;
  const size_t need = dp_workspace_bytes(problem);
  if (need > (size_t)DP_STATIC_SCRATCH_BYTES) return DP_ERR_TOO_LARGE;  // before anything touches the device
  void *ws = nullptr;
  st = static_scratch(&ws);
  if (st != DP_OK) return st;
  // every kernel of the step clears the counters it reads (no memset): what an earlier call left behind is dead
  return whole_step(problem, top_p_rule(problem, p1, p2), out, out_dtype, lse, n_exact, n_retained, n_exact_tokens,
                    ws, need, stream);
}

dp_status dp_decode_attention_timed(const dp_problem *problem, float p1, float p2, void *out, dp_dtype out_dtype,
                                    float *lse, void *workspace, size_t workspace_bytes, void *stream,
                                    void *const *events) {
  dp_status st = check_common(problem);
  if (st != DP_OK) return st;
  if (!p_in_domain(p1, p2) || !events) return DP_ERR_INVALID_ARG;
  return whole_step(problem, top_p_rule(problem, p1, p2), out, out_dtype, lse, nullptr, nullptr, nullptr, workspace,
                    workspace_bytes, stream, events);
}

dp_status dp_budget_decode_attention(const dp_problem *problem, int32_t k_retained, int32_t k_exact, void *out,
                                     dp_dtype out_dtype, float *lse, int32_t *n_exact, int32_t *n_retained,
                                     int32_t *n_exact_tokens, void *workspace, size_t workspace_bytes, void *stream) {
  dp_status st = check_common(problem);
  if (st != DP_OK) return st;
  if (k_retained < 0 || k_exact < 0) return DP_ERR_INVALID_ARG;
  return whole_step(problem, budget_rule(k_retained, k_exact), out, out_dtype, lse, n_exact, n_retained,
                    n_exact_tokens, workspace, workspace_bytes, stream);
}

dp_status dp_dense_decode(const dp_problem *problem, const int32_t *seg_rows, void *out, dp_dtype out_dtype,
                          float *lse, void *workspace, size_t workspace_bytes, void *stream) {
  if (!shape_ok(problem)) return DP_ERR_INVALID_ARG;
  if (problem->head_dim != dp::kHeadDim) return DP_ERR_UNSUPPORTED;
  if (out_dtype != DP_BF16 && out_dtype != DP_F32) return DP_ERR_UNSUPPORTED;
  if (!problem->q || !problem->seg_row_base || !seg_rows || !out || !workspace) return DP_ERR_INVALID_ARG;
  if (problem->max_rows_per_seg > 0 && (!problem->k_cache || !problem->v_cache)) return DP_ERR_INVALID_ARG;
  if (workspace_bytes < dp_workspace_bytes(problem)) return DP_ERR_WORKSPACE_TOO_SMALL;
  if (reinterpret_cast<uintptr_t>(workspace) % 256) return DP_ERR_INVALID_ARG;
  const dp::CacheView c = view_of(problem);
  const Workspace w = carve(problem, workspace);
  const dp::AttnOut attn{out, lse, out_dtype == DP_BF16};
  return dp::launch_dense(c, seg_rows, w.partials, w.splits, attn, static_cast<hipStream_t>(stream)) == hipSuccess
             ? DP_OK
             : DP_ERR_HIP;
}

static bool prefill_ok(const dp_prefill *in) {
  return in && in->n_seg >= 0 && in->total_clusters >= 0 && in->max_clusters_per_seg >= 0 &&
         in->max_rows_per_seg >= 0 && in->max_clusters_per_seg <= in->total_clusters;
}

size_t dp_build_workspace_bytes(const dp_prefill *in) {
  if (!prefill_ok(in)) return 0;
  size_t hist, rank, row_token;
  int nb;
  dp::build_workspace_layout(in->n_seg, in->max_rows_per_seg, in->max_clusters_per_seg, &hist, &rank, &row_token, &nb);
  return hist + rank + row_token;
}

dp_status dp_build_cluster_cache(const dp_prefill *in, void *k_cache, void *v_cache, int32_t *cluster_offsets,
                                 int32_t *cluster_sizes, void *k_centroids, void *v_centroids, float *v_sums,
                                 int32_t *token_row, void *workspace, size_t workspace_bytes, void *stream) {
  if (!prefill_ok(in)) return DP_ERR_INVALID_ARG;
  if (in->head_dim != dp::kHeadDim) return DP_ERR_UNSUPPORTED;
  // the per-block cluster counts of the sort live in LDS; the bound is the one the decode step has as well
  if (in->max_clusters_per_seg > dp::kSelectMaxClusters) return DP_ERR_UNSUPPORTED;
  if (in->n_seg == 0) return DP_OK;
  if (!in->seg_row_base || !in->seg_rows || !in->seg_cluster_ptr) return DP_ERR_INVALID_ARG;
  if (in->max_rows_per_seg > 0 && (!in->k_tokens || !in->v_tokens || !in->assignment || !k_cache || !v_cache))
    return DP_ERR_INVALID_ARG;
  if (in->total_clusters > 0 && (!cluster_offsets || !cluster_sizes || !k_centroids || !v_centroids))
    return DP_ERR_INVALID_ARG;
  const size_t need = dp_build_workspace_bytes(in);
  if (workspace_bytes < need) return DP_ERR_WORKSPACE_TOO_SMALL;
  if (need > 0 && (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256)) return DP_ERR_INVALID_ARG;
  dp::BuildProblem p;
  p.n_seg = in->n_seg;
  p.k_tokens = in->k_tokens;
  p.v_tokens = in->v_tokens;
  p.assignment = in->assignment;
  p.seg_row_base = in->seg_row_base;
  p.seg_rows = in->seg_rows;
  p.seg_cluster_ptr = in->seg_cluster_ptr;
  p.max_kc = in->max_clusters_per_seg;
  p.max_rows = in->max_rows_per_seg;
  p.k_cache = k_cache;
  p.v_cache = v_cache;
  p.k_centroids = k_centroids;
  p.v_centroids = v_centroids;
  p.cluster_offsets = cluster_offsets;
  p.cluster_sizes = cluster_sizes;
  p.token_row = token_row;
  p.v_sums = v_sums;
  return dp::launch_build(p, workspace, static_cast<hipStream_t>(stream)) == hipSuccess ? DP_OK : DP_ERR_HIP;
}

size_t dp_kmeans_workspace_bytes(const dp_prefill *in) {
  if (!prefill_ok(in)) return 0;
  return align_up(sizeof(float) * (size_t)in->total_clusters, 256);
}

dp_status dp_kmeans_assign(const dp_prefill *in, const void *centroids, int32_t *assignment, float *best_score,
                           void *workspace, size_t workspace_bytes, void *stream) {
  if (!prefill_ok(in)) return DP_ERR_INVALID_ARG;
  if (in->head_dim != dp::kHeadDim) return DP_ERR_UNSUPPORTED;
  if (in->n_seg == 0 || in->max_rows_per_seg == 0) return DP_OK;
  if (!in->seg_row_base || !in->seg_rows || !in->seg_cluster_ptr || !in->k_tokens || !assignment)
    return DP_ERR_INVALID_ARG;
  if (in->total_clusters > 0 && !centroids) return DP_ERR_INVALID_ARG;
  const size_t need = dp_kmeans_workspace_bytes(in);
  if (workspace_bytes < need) return DP_ERR_WORKSPACE_TOO_SMALL;
  if (need > 0 && (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256)) return DP_ERR_INVALID_ARG;
  dp::KmeansProblem p;
  p.n_seg = in->n_seg;
  p.k_tokens = in->k_tokens;
  p.centroids = centroids;
  p.seg_row_base = in->seg_row_base;
  p.seg_rows = in->seg_rows;
  p.seg_cluster_ptr = in->seg_cluster_ptr;
  p.max_rows = in->max_rows_per_seg;
  p.total_clusters = in->total_clusters;
  p.assignment = assignment;
  p.best_score = best_score;
  return dp::launch_kmeans_assign(p, static_cast<float *>(workspace), static_cast<hipStream_t>(stream)) == hipSuccess
             ? DP_OK
             : DP_ERR_HIP;
}

size_t dp_kmeans_fit_workspace_bytes(const dp_prefill *in) {
  if (!prefill_ok(in)) return 0;
  const size_t step = dp_kmeans_workspace_bytes(in) > dp_build_workspace_bytes(in) ? dp_kmeans_workspace_bytes(in)
                                                                                    : dp_build_workspace_bytes(in);
  return step + 2 * align_up(sizeof(int32_t) * (size_t)in->total_clusters, 256);
}

// Lloyd's iteration on one stream: assignment (matrix cores), then the means of the keys per cluster through the
// kernels of the cache build with nothing moved (stable counting sort of the tokens, fp64 sums in token order).
dp_status dp_kmeans_fit(const dp_prefill *in, void *centroids, int32_t n_iters, uint32_t init, int32_t *assignment,
                        float *best_score, void *workspace, size_t workspace_bytes, void *stream) {
  if (!prefill_ok(in) || n_iters < 0 || (init != DP_KMEANS_INIT_GIVEN && init != DP_KMEANS_INIT_STRIDED))
    return DP_ERR_INVALID_ARG;
  if (in->head_dim != dp::kHeadDim || in->max_clusters_per_seg > dp::kSelectMaxClusters) return DP_ERR_UNSUPPORTED;
  if (in->n_seg == 0) return DP_OK;
  if (!in->seg_row_base || !in->seg_rows || !in->seg_cluster_ptr) return DP_ERR_INVALID_ARG;
  if (in->max_rows_per_seg > 0 && (!in->k_tokens || (n_iters > 0 && !assignment))) return DP_ERR_INVALID_ARG;
  if (in->total_clusters > 0 && !centroids) return DP_ERR_INVALID_ARG;
  const size_t need = dp_kmeans_fit_workspace_bytes(in);
  if (workspace_bytes < need) return DP_ERR_WORKSPACE_TOO_SMALL;
  if (need > 0 && (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256)) return DP_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t counts = align_up(sizeof(int32_t) * (size_t)in->total_clusters, 256);
  char *ws = static_cast<char *>(workspace);
  int32_t *sizes = reinterpret_cast<int32_t *>(ws + need - 2 * counts);
  int32_t *offsets = reinterpret_cast<int32_t *>(ws + need - counts);

  dp::KmeansProblem k;
  k.n_seg = in->n_seg;
  k.k_tokens = in->k_tokens;
  k.centroids = centroids;
  k.seg_row_base = in->seg_row_base;
  k.seg_rows = in->seg_rows;
  k.seg_cluster_ptr = in->seg_cluster_ptr;
  k.max_rows = in->max_rows_per_seg;
  k.total_clusters = in->total_clusters;
  k.assignment = assignment;
  k.best_score = best_score;
  if (init == DP_KMEANS_INIT_STRIDED &&
      dp::launch_kmeans_init_strided(k, centroids, in->max_clusters_per_seg, s) != hipSuccess)
    return DP_ERR_HIP;

  dp::BuildProblem b{};
  b.n_seg = in->n_seg;
  b.k_tokens = in->k_tokens;
  b.assignment = assignment;
  b.seg_row_base = in->seg_row_base;
  b.seg_rows = in->seg_rows;
  b.seg_cluster_ptr = in->seg_cluster_ptr;
  b.max_kc = in->max_clusters_per_seg;
  b.max_rows = in->max_rows_per_seg;
  b.k_centroids = centroids;  // cache pointers null: keys only, nothing moved
  b.cluster_offsets = offsets;
  b.cluster_sizes = sizes;
  if (in->max_rows_per_seg == 0) return DP_OK;  // no tokens anywhere: nothing to assign, every centroid stays
  for (int it = 0; it < n_iters; ++it) {
    if (dp::launch_kmeans_assign(k, reinterpret_cast<float *>(ws), s) != hipSuccess) return DP_ERR_HIP;
    if (dp::launch_build(b, ws, s) != hipSuccess) return DP_ERR_HIP;
  }
  return DP_OK;
}

const char *dp_status_string(dp_status status) {
  switch (status) {
    case DP_OK: return "DP_OK";
    case DP_ERR_INVALID_ARG: return "DP_ERR_INVALID_ARG: null pointer, bad shape, p outside its domain or a negative budget";
    case DP_ERR_UNSUPPORTED: return "DP_ERR_UNSUPPORTED: head_dim != 128, GQA group > 16, too many clusters or bad dtype";
    case DP_ERR_WORKSPACE_TOO_SMALL: return "DP_ERR_WORKSPACE_TOO_SMALL: see dp_workspace_bytes";
    case DP_ERR_HIP: return "DP_ERR_HIP: a HIP runtime call failed";
    case DP_ERR_TOO_LARGE:
      return "DP_ERR_TOO_LARGE: the problem needs more scratch than DP_STATIC_SCRATCH_BYTES (use dp_decode_attention "
             "with a caller-owned workspace)";
  }
  return "unknown dp_status";
}

}  // extern "C"
