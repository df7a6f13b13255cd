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
// Work split: a head with R rows is cut into ceil(R / c) items of
// c = 64 * max(g, ceil(R / (64 * S))) rows (S = partial slots per head; g = 1..4
// grows with the launch's total rows: a light launch spreads over the whole chip
// in 64-row items, a heavy one amortises its merges, yet keeps four or more items
// per workgroup so that the last round is short: 133 us with g <= 4 against 138 us
// with g <= 8 on 1.4 M rows); item boundaries are
// multiples of 64 rows, so the first list entry of an item comes from the
// plan's chunk table in O(1).  Heads differ by orders of magnitude in
// rows and the host knows none of the counts, so the grid is a fixed number of
// workgroups that pull items from a device-side queue: every workgroup builds
// the same prefix of items per head in LDS from head_rows[], then claims item
// numbers with an atomic counter until they run out (nobody waits for anybody).
// Inside a workgroup (256 threads) each 16-lane DPP row owns one cache row per
// load (lane t holds dims [8t, 8t+8) of K for the dot and of V for the
// accumulation), keeps its own online-softmax state in base-2 exponent form,
// and the states are merged through LDS.  Partials (m, l, acc[128]) go to the
// workspace; the item of a head that finishes last (an arrival counter, no
// waiting) merges them (log-sum-exp merge), normalises and writes the output.
#include <hip/hip_ext.h>

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
constexpr int kMinItemChunks = 4;  // items of a heavy launch have at least this many 64-row chunks


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
  int32_t head0, n_heads;  // this launch serves heads [head0, head0 + n_heads), n_heads <= kMaxQueueHeads
  int32_t *queue_next;     // the launch's item counter (zeroed by the planner)
  const int32_t *pending;  // nullable: heads of this launch that have work; 0 = return at once
  // A/B variant (decode_kernel<true>): per-head buffers that hold the gathered exact rows of heads with at most rows_cap of them
  const void *k_gather, *v_gather;
  int32_t rows_cap;
  float scale_log2;        // sm_scale * log2(e)
};

// rows per item of a head with R rows (multiple of kChunkRows); g: least chunks per item of this launch
__device__ __forceinline__ int rows_per_item(int R, int S, int g) {
  return kChunkRows * max(g, (R + kChunkRows * S - 1) / (kChunkRows * S));
}

// One (head, split) item: attend its rows, publish the partial, and merge the head if this item arrives last.
template <bool kGathered>
__device__ __forceinline__ void decode_item(const DecodeArgs &a, int head, int split, int R, int g, int *s_start, int *s_src,
                                            float *s_m, float *s_l, float (*s_acc)[kHeadDim], int *s_last, int tid,
                                            int lane16, int grp) {
  const int c = rows_per_item(R, a.splits, g);
  const int row_a = split * c;
  const int row_b = min(R, row_a + c);
  const int n_active = (R + c - 1) / c;

  const int b = head / a.n_q_heads, h = head % a.n_q_heads;
  const int seg = b * a.n_kv_heads + h / a.group;
  const int c0 = a.seg_cluster_ptr[seg];
  const int n_ex = a.n_exact[head], n_rt = a.n_retained[head];
  const int32_t *ent_src = a.plan.ent_src + (int64_t)head * a.max_k;
  const int32_t *row_start = a.plan.row_start + (int64_t)head * (a.max_k + 1);

  const uint4 qv = load_row_slice(a.q, (int64_t)head, lane16);

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
  // a head whose exact rows did not fit the buffer was not gathered: it is read in place
  const bool use_gather = kGathered && n_ex > 0 && row_start[n_ex] <= a.rows_cap;
  if (use_gather) {
    src.k_gather = a.k_gather;
    src.v_gather = a.v_gather;
    src.gather_row0 = (int64_t)head * a.rows_cap;
  }

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
    // the 16 DPP-row groups take consecutive 4-row pieces: one step of the workgroup reads 64 consecutive rows
    if (use_gather)
      attend_rows<true>(st, qv, a.scale_log2, src, s_start, s_src, n_ent, ent0, n_ex, r0 + grp * kAttendBatch, r1,
                        kDecGroups * kAttendBatch, lane16);
    else
      attend_rows<false>(st, qv, a.scale_log2, src, s_start, s_src, n_ent, ent0, n_ex, r0 + grp * kAttendBatch, r1,
                         kDecGroups * kAttendBatch, lane16);
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
    (*s_last) = (ticket == n_active - 1);
  }
  __syncthreads();
  if (!(*s_last)) return;
  if (tid < kHeadDim) {
    // running log-sum-exp merge; the coherent loads of 8 partials are issued together
    float Mx = -INFINITY, Ls = 0.f, os = 0.f;
    for (int s0 = 0; s0 < n_active; s0 += 8) {
      float ms[8], ll[8], oo[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const float *Q = P + min(s0 + u, n_active - 1) * kPartialStride;
        ms[u] = __hip_atomic_load(Q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        ll[u] = __hip_atomic_load(Q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        oo[u] = __hip_atomic_load(Q + 2 + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (s0 + u < n_active) {  // every partial has a finite m: an item has at least one row
          const float Mn = fmaxf(Mx, ms[u]);
          const float sc = exp2f(Mx - Mn), w = exp2f(ms[u] - Mn);
          Ls = Ls * sc + ll[u] * w;
          os = os * sc + oo[u] * w;
          Mx = Mn;
        }
      }
    }
    store_out(a.out, a.out_is_bf16, head, tid, os / Ls);
    if (a.lse && tid == 0) a.lse[head] = (Mx + log2f(Ls)) * kLn2;
  }
}

template <bool kGathered>
__global__ __launch_bounds__(kDecThreads) void decode_kernel(DecodeArgs a) {
  __shared__ int s_start[kDecBlockRows + 1];
  __shared__ int s_src[kDecBlockRows + 1];
  __shared__ float s_m[kDecWaves], s_l[kDecWaves];
  __shared__ float s_acc[kDecWaves][kHeadDim];
  __shared__ int s_last, s_item;
  __shared__ int s_first[kMaxQueueHeads + 1];  // first item number of each head of this launch
  __shared__ int s_scan[kDecWaves + 1];
  __shared__ int s_rows[kMaxQueueHeads];
  const int tid = threadIdx.x, lane16 = tid & 15, grp = tid >> 4;
  if (a.pending && *a.pending == 0) return;  // every head was finished by the selection kernel
  // ---- the queue: items per head from head_rows[], exclusive prefix in LDS ----
  constexpr int kPer = kMaxQueueHeads / kDecThreads;  // consecutive heads per thread
  int rows[kPer], chunks = 0;
#pragma unroll
  for (int u = 0; u < kPer; ++u) {
    const int hh = tid * kPer + u;
    rows[u] = hh < a.n_heads ? a.plan.head_rows[a.head0 + hh] : 0;  // <= 0: nothing to do (empty, or attended already)
    s_rows[hh] = rows[u];
    if (rows[u] > 0) chunks += min(1 << 20, (rows[u] + kChunkRows - 1) / kChunkRows);  // capped: the sum stays in range
  }
  // least chunks per item: about one item for every second workgroup of the grid, between 1 and kMinItemChunks
  const int all_chunks = block_sum<int, kDecWaves>(chunks, s_scan);
  const int g = min(kMinItemChunks, max(1, (all_chunks + kDecodeGrid / 2 - 1) / (kDecodeGrid / 2)));
  int cnt[kPer], mine = 0;
#pragma unroll
  for (int u = 0; u < kPer; ++u) {
    int n = 0;
    if (rows[u] > 0) {
      const int c = rows_per_item(rows[u], a.splits, g);
      n = (rows[u] + c - 1) / c;
    }
    cnt[u] = n;
    mine += n;
  }
  int total;
  int run = block_excl_scan<int, kDecWaves>(mine, s_scan, total);
#pragma unroll
  for (int u = 0; u < kPer; ++u) {
    s_first[tid * kPer + u] = run;
    run += cnt[u];
  }
  if (tid == kDecThreads - 1) s_first[kMaxQueueHeads] = total;
  __syncthreads();
  if (total == 0) return;

#pragma unroll 1
  // the first item of a workgroup is its block index; further items are claimed from the counter
  for (int item = blockIdx.x; item < total;) {
    // head that owns the item: the largest hh with s_first[hh] <= item (heads without items repeat the
    // next head's value, so the largest such hh is the one with s_first[hh + 1] > item)
    int lo = 0, hi = kMaxQueueHeads;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (s_first[mid] <= item) lo = mid; else hi = mid;
    }
    const int head = a.head0 + lo, split = item - s_first[lo];
    decode_item<kGathered>(a, head, split, s_rows[lo], g, s_start, s_src, s_m, s_l, s_acc, &s_last, tid, lane16, grp);
    if (total <= (int)gridDim.x) break;  // every item had its workgroup: nothing to claim
    if (tid == 0)
      s_item = gridDim.x + __hip_atomic_fetch_add(a.queue_next, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();  // also: LDS is reused by the next item
    item = s_item;
    __syncthreads();
  }
}

}  // namespace


hipError_t launch_decode(const CacheView &c, const int32_t *n_exact, const int32_t *n_retained, const Plan &plan,
                         float *partials, int splits, const AttnOut &attn, hipStream_t s, hipEvent_t start,
                         hipEvent_t stop, const void *k_gather, const void *v_gather, int rows_cap) {
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
  a.k_gather = k_gather;
  a.v_gather = v_gather;
  a.rows_cap = rows_cap;
  // one launch per slab of kMaxQueueHeads heads, each with its own item counter
  for (int h0 = 0, slab = 0; h0 < nh; h0 += kMaxQueueHeads, ++slab) {
    a.head0 = h0;
    a.n_heads = nh - h0 < kMaxQueueHeads ? nh - h0 : kMaxQueueHeads;
    a.queue_next = plan.queue_next + slab;
    a.pending = plan.pending ? plan.pending + slab : nullptr;
    const long max_items = (long)a.n_heads * splits;
    const int grid = (int)(max_items < kDecodeGrid ? max_items : kDecodeGrid);
    // measurement: the events bracket the first slab's begin and the last slab's end
    hipEvent_t ev0 = (h0 == 0) ? start : nullptr, ev1 = (h0 + kMaxQueueHeads >= nh) ? stop : nullptr;
    if (k_gather)
      hipLaunchKernelGGL(decode_kernel<true>, dim3(grid), dim3(kDecThreads), 0, s, a);
    else if (ev0 || ev1)
      hipExtLaunchKernelGGL(decode_kernel<false>, dim3(grid), dim3(kDecThreads), 0, s, ev0, ev1, 0, a);
    else
      hipLaunchKernelGGL(decode_kernel<false>, dim3(grid), dim3(kDecThreads), 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace dp
