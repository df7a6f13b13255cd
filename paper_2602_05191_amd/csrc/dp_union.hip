// A/B variant: selection per GQA group.  The paper states the method for one
// query; with grouped-query attention (its model has groups of 4, Sec. 5.1) the
// two top-p sets can be taken per query head (the product path) or per group.
// This variant takes them per head as usual and then lets every head of a group
// attend over the UNION of the group's sets:
//   exact(group)  = union over the heads of their exact sets
//   approx(group) = (union of their retained sets) minus exact(group)
// so that a K / V row is read once for the whole group (as the dense kernel reads
// it) instead of once per head that selected it.  Every head attends a superset
// of its own selection: the result is NOT the per-head method's (it lies between
// it and dense attention); the variant exists to measure what sharing the reads
// buys and what the extra rows per head cost.
//
//   union_kernel          one workgroup per segment: marks the heads' lists in an
//                         LDS bit table (2 bits per cluster), compacts both sets in
//                         ascending cluster index
//   (plan_kernel of the selection file, with segments in the place of heads)
//   group_decode_kernel   one workgroup per (segment, split): walks the union row
//                         list once, scores every row against the G heads from
//                         registers (one online-softmax state per head and DPP row)
//   group_merge_kernel    log-sum-exp merge of the splits, one workgroup per head
#include "dp_attend.hpp"
#include "dp_device.hpp"
#include "dp_kernels.hpp"

namespace dp {
namespace {

constexpr int kUnionThreads = 1024;
constexpr int kUnionWaves = kUnionThreads / 64;

struct UnionArgs {
  const int32_t *seg_cluster_ptr;
  const int32_t *sel_ids, *n_exact, *n_retained;  // per head
  int32_t *union_ids, *n_exact_u, *n_retained_u;  // per segment
  int32_t n_kv_heads, n_q_heads, group, max_k;
};

__global__ __launch_bounds__(kUnionThreads) void union_kernel(UnionArgs a) {
  __shared__ uint32_t s_bits[kGroupUnionMaxClusters / 16];  // cluster i: bit 2 (i % 16) retained, bit 2 (i % 16) + 1 exact
  __shared__ int s_scan[2 * (kUnionWaves + 1)];
  const int seg = blockIdx.x, tid = threadIdx.x;
  const int b = seg / a.n_kv_heads, g = seg % a.n_kv_heads;
  const int kc = a.seg_cluster_ptr[seg + 1] - a.seg_cluster_ptr[seg];
  const int n_words = (kc + 15) / 16;
  for (int i = tid; i < n_words; i += kUnionThreads) s_bits[i] = 0;
  __syncthreads();
  for (int h = 0; h < a.group; ++h) {
    const int64_t head = (int64_t)b * a.n_q_heads + g * a.group + h;
    const int ne = a.n_exact[head], nr = a.n_retained[head];
    const int32_t *sel = a.sel_ids + head * a.max_k;
    for (int j = tid; j < nr; j += kUnionThreads) {
      const int id = sel[j];
      if (id >= 0 && id < kc) atomicOr(&s_bits[id >> 4], (j < ne ? 3u : 1u) << (2 * (id & 15)));
    }
  }
  __syncthreads();
  // compaction in ascending cluster index: thread t owns words [t * per, (t + 1) * per)
  const int per = (n_words + kUnionThreads - 1) / kUnionThreads;
  const int w0 = min(n_words, tid * per), w1 = min(n_words, w0 + per);
  int ce = 0, ca = 0;
  for (int w = w0; w < w1; ++w) {
    const uint32_t v = s_bits[w];
    const uint32_t ex = (v >> 1) & 0x55555555u, rt = v & 0x55555555u;
    ce += __popc(ex);
    ca += __popc(rt & ~ex);
  }
  int n_ex, n_ap;
  int pe = block_excl_scan<int, kUnionWaves>(ce, s_scan, n_ex);
  int pa = block_excl_scan<int, kUnionWaves>(ca, s_scan, n_ap);
  int32_t *out = a.union_ids + (int64_t)seg * a.max_k;
  for (int w = w0; w < w1; ++w) {
    const uint32_t v = s_bits[w];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const uint32_t two = (v >> (2 * u)) & 3u;
      if (two & 2u) out[pe++] = w * 16 + u;
      else if (two & 1u) out[n_ex + pa++] = w * 16 + u;
    }
  }
  if (tid == 0) {
    a.n_exact_u[seg] = n_ex;
    a.n_retained_u[seg] = n_ex + n_ap;
  }
}

// ---- one pass over the union row list for GH heads of the group ----
constexpr int kGrpThreads = 256;
constexpr int kGrpWaves = kGrpThreads / 64;
constexpr int kGrpGroups = kGrpThreads / 16;
constexpr int kGrpBlockRows = 512;  // rows resolved per LDS staging round
constexpr int kGrpPartialStride = kHeadDim + 2;  // m, l, acc[128]

struct GroupArgs {
  const void *q, *k_cache, *v_cache, *k_centroids, *v_centroids;
  const int64_t *seg_row_base;
  const int32_t *seg_cluster_ptr, *cluster_sizes;
  const int32_t *n_exact_u, *n_retained_u;  // per segment
  Plan plan;                                // per segment (segments in the place of heads)
  float *partials;                          // [n_seg, splits, group, kGrpPartialStride]
  void *out;
  float *lse;
  int32_t out_is_bf16;
  int32_t n_kv_heads, n_q_heads, group, max_k, splits, head0;
  float scale_log2;
};

// rows per split of a segment with R rows: a multiple of the chunk size
__device__ __forceinline__ int group_rows_per_split(int R, int S) {
  return kChunkRows * max(1, (R + kChunkRows * S - 1) / (kChunkRows * S));
}

// The row walk of attend_rows for GH heads at once: rows ra .. ra+B-1, ra+stride .., below rb.
template <int GH>
__device__ __forceinline__ void attend_rows_group(RowState (&st)[GH], const uint4 (&qv)[GH], float scale_log2,
                                                  const RowSources &src, const int *s_start, const int *s_src,
                                                  int n_ent, int ent0, int n_ex, int ra, int rb, int stride,
                                                  int lane16) {
  if (ra >= rb) return;
  int k = 0;  // entry that holds row ra: largest k in [0, n_ent) with s_start[k] <= ra
  {
    int hi = n_ent;
    while (hi - k > 1) {
      const int mid = (k + hi) >> 1;
      if (s_start[mid] <= ra) k = mid; else hi = mid;
    }
  }
  int next_start = s_start[k + 1];
  for (int r = ra; r < rb; r += stride) {
    uint4 kraw[kAttendBatch], vraw[kAttendBatch];
    float beta[kAttendBatch];  // additive weight of the row (base 2); -inf: no row
#pragma unroll
    for (int u = 0; u < kAttendBatch; ++u) {
      const int row = r + u;
      beta[u] = -INFINITY;
      kraw[u] = make_uint4(0, 0, 0, 0);
      vraw[u] = make_uint4(0, 0, 0, 0);
      if (row < rb) {
        while (row >= next_start) {  // walk forward to the entry that holds this row
          ++k;
          next_start = s_start[k + 1];
        }
        const int s = s_src[k];
        if (ent0 + k < n_ex) {
          const int64_t g = src.seg_row0 + s + (row - s_start[k]);
          kraw[u] = load_row_slice(src.k_cache, g, lane16);
          vraw[u] = load_row_slice(src.v_cache, g, lane16);
          beta[u] = 0.f;
        } else {
          kraw[u] = load_row_slice(src.k_centroids, src.c0 + s, lane16);
          vraw[u] = load_row_slice(src.v_centroids, src.c0 + s, lane16);
          beta[u] = log2f((float)src.seg_sizes[s]);
        }
      }
    }
    float vf[kAttendBatch][8];
#pragma unroll
    for (int u = 0; u < kAttendBatch; ++u) unpack8(vraw[u], vf[u]);
#pragma unroll
    for (int j = 0; j < GH; ++j) {
      float x[kAttendBatch];
      float m_new = st[j].m;
#pragma unroll
      for (int u = 0; u < kAttendBatch; ++u) {
        const float d = row16_sum(dot8_bf16(qv[j], kraw[u])) * scale_log2;
        x[u] = beta[u] == -INFINITY ? -INFINITY : d + beta[u];
        m_new = fmaxf(m_new, x[u]);
      }
      // m_new is finite here: row r is a row of the list
      const float alpha = exp2f(st[j].m - m_new);  // st.m = -inf gives 0
      st[j].l *= alpha;
#pragma unroll
      for (int i = 0; i < 8; ++i) st[j].acc[i] *= alpha;
#pragma unroll
      for (int u = 0; u < kAttendBatch; ++u) {
        const float p = exp2f(x[u] - m_new);
        st[j].l += p;
#pragma unroll
        for (int i = 0; i < 8; ++i) st[j].acc[i] = fmaf(p, vf[u][i], st[j].acc[i]);
      }
      st[j].m = m_new;
    }
  }
}

template <int GH>
__global__ __launch_bounds__(kGrpThreads) void group_decode_kernel(GroupArgs a) {
  __shared__ int s_start[kGrpBlockRows + 1];
  __shared__ int s_src[kGrpBlockRows + 1];
  __shared__ float s_m[kGrpWaves], s_l[kGrpWaves];
  __shared__ float s_acc[kGrpWaves][kHeadDim];
  const int seg = blockIdx.y, split = blockIdx.x;
  const int tid = threadIdx.x, lane16 = tid & 15, grp = tid >> 4;
  const int R = a.plan.head_rows[seg];
  if (R <= 0) return;
  const int c = group_rows_per_split(R, a.splits);
  const int row_a = split * c;
  if (row_a >= R) return;
  const int row_b = min(R, row_a + c);

  const int b = seg / a.n_kv_heads, g = seg % a.n_kv_heads;
  const int c0 = a.seg_cluster_ptr[seg];
  const int n_ex = a.n_exact_u[seg], n_rt = a.n_retained_u[seg];
  const int32_t *ent_src = a.plan.ent_src + (int64_t)seg * a.max_k;
  const int32_t *row_start = a.plan.row_start + (int64_t)seg * (a.max_k + 1);

  uint4 qv[GH];
#pragma unroll
  for (int j = 0; j < GH; ++j)
    qv[j] = load_row_slice(a.q, (int64_t)b * a.n_q_heads + g * a.group + a.head0 + j, lane16);

  RowSources src;
  src.k_cache = a.k_cache;
  src.v_cache = a.v_cache;
  src.k_centroids = a.k_centroids;
  src.v_centroids = a.v_centroids;
  src.seg_sizes = a.cluster_sizes + c0;
  src.seg_row0 = a.seg_row_base[seg];
  src.c0 = c0;
  src.k_gather = src.v_gather = nullptr;
  src.gather_row0 = 0;

  RowState st[GH];
#pragma unroll
  for (int j = 0; j < GH; ++j) row_state_init(st[j]);

  int ent0 = a.plan.chunk_entry[(int64_t)seg * a.plan.chunk_stride + row_a / kChunkRows];
  for (int r0 = row_a; r0 < row_b; r0 += kGrpBlockRows) {
    const int r1 = min(row_b, r0 + kGrpBlockRows);
    // stage the list entries that cover rows [r0, r1): every entry has >= 1 row
    const int n_ent = min(r1 - r0, n_rt - ent0);
    __syncthreads();
    for (int k = tid; k <= n_ent; k += kGrpThreads) {
      s_start[k] = row_start[ent0 + k];
      s_src[k] = (k < n_ent) ? ent_src[ent0 + k] : 0;
    }
    __syncthreads();
    attend_rows_group<GH>(st, qv, a.scale_log2, src, s_start, s_src, n_ent, ent0, n_ex, r0 + grp * kAttendBatch, r1,
                          kGrpGroups * kAttendBatch, lane16);
    if (r1 < row_b) {  // first entry of the next block: the entry that holds row r1
      int lo = 0, hi = n_ent + 1;  // s_start[n_ent] is staged as well
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (s_start[mid] <= r1) lo = mid; else hi = mid;
      }
      ent0 += lo;
    }
  }
  // one partial per head of the pass
#pragma unroll
  for (int j = 0; j < GH; ++j) {
    float M, L, o;
    __syncthreads();  // the LDS of the previous merge (or of the staging) has been read by everybody
    block_merge<kGrpWaves>(st[j], s_m, s_l, s_acc, kGrpWaves, M, L, o);
    if (tid < kHeadDim) {
      float *P = a.partials + (((int64_t)seg * a.splits + split) * a.group + a.head0 + j) * kGrpPartialStride;
      if (tid == 0) {
        P[0] = M;
        P[1] = L;
      }
      P[2 + tid] = o;
    }
  }
}

__global__ __launch_bounds__(kHeadDim) void group_merge_kernel(GroupArgs a) {
  const int head = blockIdx.x, tid = threadIdx.x;
  const int b = head / a.n_q_heads, h = head % a.n_q_heads;
  const int seg = b * a.n_kv_heads + h / a.group, j = h % a.group;
  const int R = a.plan.head_rows[seg];
  if (R <= 0) {  // nothing selected in the whole group: zero output
    store_out(a.out, a.out_is_bf16, head, tid, 0.f);
    if (a.lse && tid == 0) a.lse[head] = -INFINITY;
    return;
  }
  const int c = group_rows_per_split(R, a.splits);
  const int n_active = (R + c - 1) / c;
  float M = -INFINITY, L = 0.f, o = 0.f;
  for (int s = 0; s < n_active; ++s) {  // every active split holds at least one row: its m is finite
    const float *P = a.partials + (((int64_t)seg * a.splits + s) * a.group + j) * kGrpPartialStride;
    const float m = P[0];
    const float Mn = fmaxf(M, m);
    const float sc = exp2f(M - Mn), w = exp2f(m - Mn);
    L = L * sc + P[1] * w;
    o = o * sc + P[2 + tid] * w;
    M = Mn;
  }
  store_out(a.out, a.out_is_bf16, head, tid, o / L);
  if (a.lse && tid == 0) a.lse[head] = (M + log2f(L)) * kLn2;
}

}  // namespace

hipError_t launch_group_union(const CacheView &c, const int32_t *sel_ids, const int32_t *n_exact,
                              const int32_t *n_retained, int32_t *union_ids, int32_t *n_exact_u,
                              int32_t *n_retained_u, hipStream_t s) {
  const int n_seg = c.batch * c.n_kv_heads;
  if (n_seg == 0) return hipSuccess;
  if (c.max_clusters_per_seg > kGroupUnionMaxClusters) return hipErrorInvalidValue;
  UnionArgs a;
  a.seg_cluster_ptr = c.seg_cluster_ptr;
  a.sel_ids = sel_ids;
  a.n_exact = n_exact;
  a.n_retained = n_retained;
  a.union_ids = union_ids;
  a.n_exact_u = n_exact_u;
  a.n_retained_u = n_retained_u;
  a.n_kv_heads = c.n_kv_heads;
  a.n_q_heads = c.n_q_heads;
  a.group = c.group;
  a.max_k = c.max_clusters_per_seg;
  hipLaunchKernelGGL(union_kernel, dim3(n_seg), dim3(kUnionThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_group_decode(const CacheView &c, const int32_t *n_exact_u, const int32_t *n_retained_u,
                               const Plan &seg_plan, float *partials, int splits, const AttnOut &attn, hipStream_t s) {
  const int n_seg = c.batch * c.n_kv_heads, nh = c.batch * c.n_q_heads;
  if (nh == 0) return hipSuccess;
  GroupArgs a;
  a.q = c.q;
  a.k_cache = c.k_cache;
  a.v_cache = c.v_cache;
  a.k_centroids = c.k_centroids;
  a.v_centroids = c.v_centroids;
  a.seg_row_base = c.seg_row_base;
  a.seg_cluster_ptr = c.seg_cluster_ptr;
  a.cluster_sizes = c.cluster_sizes;
  a.n_exact_u = n_exact_u;
  a.n_retained_u = n_retained_u;
  a.plan = seg_plan;
  a.partials = partials;
  a.out = attn.out;
  a.lse = attn.lse;
  a.out_is_bf16 = attn.out_is_bf16;
  a.n_kv_heads = c.n_kv_heads;
  a.n_q_heads = c.n_q_heads;
  a.group = c.group;
  a.max_k = c.max_clusters_per_seg;
  a.splits = splits;
  a.scale_log2 = c.sm_scale * kLog2e;
  const dim3 grid(splits, n_seg);
  // the heads of a group 8 / 4 / 2 / 1 at a time (one pass over the rows when G is 1, 2, 4 or 8)
  for (int h0 = 0; h0 < c.group;) {
    const int left = c.group - h0, gh = left >= 8 ? 8 : left >= 4 ? 4 : left >= 2 ? 2 : 1;
    a.head0 = h0;
    switch (gh) {
      case 8: hipLaunchKernelGGL(group_decode_kernel<8>, grid, dim3(kGrpThreads), 0, s, a); break;
      case 4: hipLaunchKernelGGL(group_decode_kernel<4>, grid, dim3(kGrpThreads), 0, s, a); break;
      case 2: hipLaunchKernelGGL(group_decode_kernel<2>, grid, dim3(kGrpThreads), 0, s, a); break;
      default: hipLaunchKernelGGL(group_decode_kernel<1>, grid, dim3(kGrpThreads), 0, s, a); break;
    }
    h0 += gh;
  }
  hipLaunchKernelGGL(group_merge_kernel, dim3(nh), dim3(kHeadDim), 0, s, a);
  return hipGetLastError();
}

}  // namespace dp
