// Stage 3: fused gather + weighted flash-decode + split combine
// (paper Sec. 4.3 Eq. 8 and Eq. 9; the "weighted attention" of Sec. 4.4).
//
// A head's work is a list of rows: the tokens of its exact clusters (K row,
// V row, additive weight 0) followed by one pseudo-token per approximated
// cluster (key-centroid row, mean-value row, additive weight ln s_i, which
// makes its softmax weight s_i * exp(xbar_i) = Zhat_i).  Rows are read IN
// PLACE from the cluster-contiguous cache: no gather buffer is materialised, so
// the traffic is the 512 B per row the method itself needs.
//
// Work split: head x split.  A head with R rows uses ceil(R / c) splits of
// c = 64 * ceil(R / (64 * S)) rows; split boundaries are multiples of 64 rows
// so the first list entry of a split comes from the plan's chunk table in O(1).
// Inside a workgroup (256 threads) each 16-lane DPP row owns one cache row per
// load (lane t holds dims [8t, 8t+8) of K for the dot and of V for the
// accumulation), keeps its own online-softmax state in base-2 exponent form,
// and the states are merged through LDS.  Partials (m, l, acc[128]) go to the
// workspace; the split of a head that finishes last (an arrival counter, no
// waiting) merges them (log-sum-exp merge), normalises and writes the output.
#include "dp_attend.hpp"
#include "dp_device.hpp"
#include "dp_kernels.hpp"

namespace dp {
namespace {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / 64;
constexpr int kDecGroups = kDecThreads / 16;   // 16 DPP rows per workgroup
constexpr int kDecBlockRows = 512;             // rows resolved per LDS staging round
constexpr int kPartialStride = kHeadDim + 2;   // m, l, acc[128]

struct DecodeArgs {
  const void *q, *k_cache, *v_cache, *k_centroids, *v_centroids;
  const int64_t *seg_row_base;
  const int32_t *seg_cluster_ptr, *cluster_sizes;
  const int32_t *n_exact, *n_retained;
  Plan plan;
  float *partials;
  void *out;
  float *lse;  // nullable
  int32_t n_kv_heads, n_q_heads, group, max_k, splits, out_is_bf16;
  float scale_log2;  // sm_scale * log2(e)
};

// rows per split of a head with R rows (multiple of kChunkRows)
__device__ __forceinline__ int rows_per_split(int R, int S) {
  return kChunkRows * ((R + kChunkRows * S - 1) / (kChunkRows * S));
}

__global__ __launch_bounds__(kDecThreads) void decode_kernel(DecodeArgs a) {
  __shared__ int s_start[kDecBlockRows + 1];
  __shared__ int s_src[kDecBlockRows + 1];
  __shared__ float s_m[kDecWaves], s_l[kDecWaves];
  __shared__ float s_acc[kDecWaves][kHeadDim];
  __shared__ int s_last;

  const int head = blockIdx.y, split = blockIdx.x;
  const int R = a.plan.head_rows[head];
  if (R <= 0) return;  // 0: no rows (output already written); -1: attended by the selection kernel
  const int c = rows_per_split(R, a.splits);
  const int row_a = split * c;
  if (row_a >= R) return;
  const int row_b = min(R, row_a + c);
  const int n_active = (R + c - 1) / c;

  const int b = head / a.n_q_heads, h = head % a.n_q_heads;
  const int seg = b * a.n_kv_heads + h / a.group;
  const int c0 = a.seg_cluster_ptr[seg];
  const int n_ex = a.n_exact[head], n_rt = a.n_retained[head];
  const int32_t *ent_src = a.plan.ent_src + (int64_t)head * a.max_k;
  const int32_t *row_start = a.plan.row_start + (int64_t)head * (a.max_k + 1);
  const int tid = threadIdx.x, lane16 = tid & 15, grp = tid >> 4;

  const uint4 qv = load_row_slice(a.q, (int64_t)head, lane16);

  RowSources src;
  src.k_cache = a.k_cache;
  src.v_cache = a.v_cache;
  src.k_centroids = a.k_centroids;
  src.v_centroids = a.v_centroids;
  src.seg_sizes = a.cluster_sizes + c0;
  src.seg_row0 = a.seg_row_base[seg];
  src.c0 = c0;

  RowState st;
  row_state_init(st);

  int ent0 = a.plan.chunk_entry[(int64_t)head * a.plan.chunk_stride + row_a / kChunkRows];

  for (int r0 = row_a; r0 < row_b; r0 += kDecBlockRows) {
    const int r1 = min(row_b, r0 + kDecBlockRows);
    // stage the list entries that cover rows [r0, r1): every entry has >= 1 row
    const int n_ent = min(r1 - r0, n_rt - ent0);
    __syncthreads();
    for (int k = tid; k <= n_ent; k += kDecThreads) {
      s_start[k] = row_start[ent0 + k];
      s_src[k] = (k < n_ent) ? ent_src[ent0 + k] : 0;
    }
    __syncthreads();
    // each DPP-row group streams a contiguous run of the block's rows
    const int per = kAttendBatch * ((r1 - r0 + kDecGroups * kAttendBatch - 1) / (kDecGroups * kAttendBatch));
    const int ra = r0 + grp * per;
    attend_rows(st, qv, a.scale_log2, src, s_start, s_src, n_ent, ent0, n_ex, ra, min(r1, ra + per), lane16);
    // first entry of the next block: the entry that holds row r1
    if (r1 < row_b) {
      int lo = 0, hi = n_ent + 1;  // s_start[n_ent] is staged as well
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (s_start[mid] <= r1) lo = mid; else hi = mid;
      }
      ent0 += lo;
    }
  }

  float M, L, o;
  block_merge<kDecWaves>(st, s_m, s_l, s_acc, kDecWaves, M, L, o);

  if (n_active == 1) {  // the only split of this head: finish here
    if (tid < kHeadDim) {
      store_out(a.out, a.out_is_bf16, head, tid, o / L);
      if (a.lse && tid == 0) a.lse[head] = (M + log2f(L)) * kLn2;
    }
    return;
  }

  // Partials are exchanged through device-coherent (agent-scope) stores and loads, which go
  // straight to memory: no L2 write-back or invalidate of the whole cache is needed around the
  // arrival counter, only "my stores have completed" before the ticket is taken.
  float *P = a.partials + (int64_t)head * a.splits * kPartialStride;
  if (tid < kHeadDim) {
    float *mine = P + (int64_t)split * kPartialStride;
    if (tid == 0) {
      __hip_atomic_store(mine + 0, M, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(mine + 1, L, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __hip_atomic_store(mine + 2 + tid, o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __builtin_amdgcn_s_waitcnt(0);  // all of this thread's memory operations have completed
  __syncthreads();
  // The split that arrives last merges all partials of the head (log-sum-exp merge).
  if (tid == 0) {
    const int ticket = __hip_atomic_fetch_add(&a.plan.done[head], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = (ticket == n_active - 1);
  }
  __syncthreads();
  if (!s_last) return;
  if (tid < kHeadDim) {
    float Mx = -INFINITY;
    for (int s2 = 0; s2 < n_active; ++s2)
      Mx = fmaxf(Mx, __hip_atomic_load(P + s2 * kPartialStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    float Ls = 0.f, os = 0.f;
    for (int s2 = 0; s2 < n_active; ++s2) {
      const float *Q = P + s2 * kPartialStride;
      const float ms = __hip_atomic_load(Q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const float w = exp2f(ms - Mx);
      Ls += __hip_atomic_load(Q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) * w;
      os += __hip_atomic_load(Q + 2 + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) * w;
    }
    store_out(a.out, a.out_is_bf16, head, tid, os / Ls);
    if (a.lse && tid == 0) a.lse[head] = (Mx + log2f(Ls)) * kLn2;
  }
}

}  // namespace

hipError_t launch_decode(const CacheView &c, const int32_t *n_exact, const int32_t *n_retained, const Plan &plan,
                         float *partials, int splits, const AttnOut &attn, hipStream_t s) {
  const int nh = c.batch * c.n_q_heads;
  if (nh == 0) return hipSuccess;
  DecodeArgs a;
  a.q = c.q;
  a.k_cache = c.k_cache;
  a.v_cache = c.v_cache;
  a.k_centroids = c.k_centroids;
  a.v_centroids = c.v_centroids;
  a.seg_row_base = c.seg_row_base;
  a.seg_cluster_ptr = c.seg_cluster_ptr;
  a.cluster_sizes = c.cluster_sizes;
  a.n_exact = n_exact;
  a.n_retained = n_retained;
  a.plan = plan;
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
  hipLaunchKernelGGL(decode_kernel, dim3(splits, nh), dim3(kDecThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace dp
