// Stage 3 as device code: fused gather + weighted flash-decode + split combine
// (paper Sec. 4.3 Eq. 8 and Eq. 9; the "weighted attention" of Sec. 4.4), shared by
// the decode kernel (dp_decode.hip) and by the selection kernel, which runs the
// same queue after its own selections when a launch serves few heads.
//
// A head's work is a list of rows: the tokens of its exact clusters (K row,
// V row, additive weight 0) followed by one pseudo-token per approximated
// cluster (key-centroid row, mean-value row, additive weight ln s_i, which
// makes its softmax weight s_i * exp(xbar_i) = Zhat_i).  Rows are read IN
// PLACE from the cluster-contiguous cache: no gather buffer is materialised, so
// the traffic is the 512 B per row the method itself needs.
//
// Work split: a head with R rows is cut into ceil(R / c) items of
// c = 64 * max(g, ceil(R / (64 * S))) rows (S = partial slots per head; g grows
// with the launch's total rows up to the rows one workgroup step covers: a light
// launch spreads over the whole chip in small items, a heavy one amortises its
// merges, yet keeps several items per workgroup so that the last round is short).
// Item boundaries are multiples of 64 rows, so the first list entry of an item
// comes from the plan's chunk table in O(1).  Heads differ by orders of magnitude
// in rows and the host knows none of the counts, so the grid is a fixed number of
// workgroups that pull items from a device-side queue: every workgroup builds
// the same prefix of items per head in LDS from head_rows[], then claims item
// numbers with an atomic counter until they run out (nobody waits for anybody).
// Inside a workgroup of T threads each 16-lane DPP row owns one cache row per
// load (lane t holds dims [8t, 8t+8) of K for the dot and of V for the
// accumulation), keeps its own online-softmax state in base-2 exponent form,
// and the states are merged through LDS.  Partials (m, l, acc[128]) go to the
// workspace; the item of a head that finishes last (an arrival counter, no
// waiting) merges them (log-sum-exp merge), normalises and writes the output.
#pragma once

#include "dp_attend.hpp"
#include "dp_device.hpp"
#include "dp_kernels.hpp"

namespace dp {

constexpr int kPartialStride = kHeadDim + 2;  // m, l, acc[128]

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
  int32_t *queue_next;     // the launch's item counter (zeroed before the first claim)
  const int32_t *pending;  // nullable: heads of this launch that have work; 0 = return at once
  // A/B variant (kGathered): per-head buffers that hold the gathered exact rows of heads with at most rows_cap of them
  const void *k_gather, *v_gather;
  int32_t rows_cap;
  float scale_log2;  // sm_scale * log2(e)
};

// everything but the launch's slice of heads and its counters (head0, n_heads, queue_next, pending)
inline DecodeArgs decode_args_of(const CacheView &c, const int32_t *n_exact, const int32_t *n_retained,
                                 const Plan &plan, float *partials, int splits, const AttnOut &attn) {
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
  a.k_gather = a.v_gather = nullptr;
  a.rows_cap = 0;
  a.head0 = 0;
  a.n_heads = 0;
  a.queue_next = nullptr;
  a.pending = nullptr;
  return a;
}

// An int32 that another workgroup of the SAME launch may have written (kCoherent, a template parameter in scope):
// a device-coherent load that does not hit a stale line of this compute die's L2; data of an earlier launch is read
// with a plain load.  (A macro: through a function the plain loads of uniform addresses were no longer scalar loads,
// eight more vector registers and a wave of occupancy on the decode kernel.)
#define DP_LD_I32(lvalue) \
  (kCoherent ? __hip_atomic_load(&(lvalue), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : (lvalue))

// Rows in flight per 16-lane row in the queue.  Inside the selection's launch a CU holds one or two large
// workgroups (16 waves at most, against 20 of the decode kernel's small ones), and every barrier of an item stops all
// of them: the rows in flight per wave are doubled there (32 flat heads over 128 k tokens: 105 -> 98 us per step).
__host__ __device__ constexpr int queue_batch(bool coherent) { return coherent ? 8 : kAttendBatch; }

// rows per item of a head with R rows (multiple of kChunkRows); g: least chunks per item of this launch
__device__ __forceinline__ int rows_per_item(int R, int S, int g) {
  return kChunkRows * max(g, (R + kChunkRows * S - 1) / (kChunkRows * S));
}

// LDS of the queue, declared by the kernel that runs it (separate arrays: as members of one struct the same code
// needed 16 more vector registers and lost a wave of occupancy on the decode kernel)
#define DP_DECODE_LDS(T)                                                                           \
  __shared__ int s_start[((T) > 512 ? (T) : 512) + 1]; /* rows resolved per LDS staging round */    \
  __shared__ int s_src[((T) > 512 ? (T) : 512) + 1];                                               \
  __shared__ float s_m[(T) / 64], s_l[(T) / 64];                                                   \
  __shared__ float s_acc[(T) / 64][kHeadDim];                                                      \
  __shared__ int s_last, s_item;                                                                   \
  __shared__ int s_first[kMaxQueueHeads + 1]; /* first item number of each head of this launch */  \
  __shared__ int s_scan[(T) / 64 + 1];                                                             \
  __shared__ int s_rows[kMaxQueueHeads]
#define DP_DECODE_LDS_ARGS s_start, s_src, s_m, s_l, s_acc, &s_last, &s_item, s_first, s_scan, s_rows

// One (head, split) item: attend its rows, publish the partial, and merge the head if this item arrives last.
template <int T, bool kGathered, bool kCoherent>
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
  const int n_ex = DP_LD_I32(a.n_exact[head]), n_rt = DP_LD_I32(a.n_retained[head]);
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

  int ent0 = DP_LD_I32(a.plan.chunk_entry[(int64_t)head * a.plan.chunk_stride + row_a / kChunkRows]);

  for (int r0 = row_a; r0 < row_b; r0 += (T > 512 ? T : 512)) {
    const int r1 = min(row_b, r0 + (T > 512 ? T : 512));
    // stage the list entries that cover rows [r0, r1): every entry has >= 1 row
    const int n_ent = min(r1 - r0, n_rt - ent0);
    __syncthreads();
    for (int k = tid; k <= n_ent; k += T) {
      if (!kCoherent) {  // both loads go out together (n_ent >= 1: an item has a row)
        const int start = row_start[ent0 + k];
        const int source = ent_src[ent0 + min(k, n_ent - 1)];
        s_start[k] = start;
        s_src[k] = (k < n_ent) ? source : 0;
      } else {
        s_start[k] = DP_LD_I32(row_start[ent0 + k]);
        s_src[k] = (k < n_ent) ? DP_LD_I32(ent_src[ent0 + k]) : 0;
      }
    }
    __syncthreads();
    // the DPP-row groups take consecutive pieces of kB rows: one step of the workgroup reads T / 16 * kB consecutive
    // rows
    constexpr int kB = queue_batch(kCoherent);
    if (use_gather)
      attend_rows<true, kB>(st, qv, a.scale_log2, src, s_start, s_src, n_ent, ent0, n_ex, r0 + grp * kB, r1,
                            (T / 16) * kB, lane16);
    else
      attend_rows<false, kB>(st, qv, a.scale_log2, src, s_start, s_src, n_ent, ent0, n_ex, r0 + grp * kB, r1,
                             (T / 16) * kB, lane16);
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
  // (waves beyond the item's rows hold the empty state: a large workgroup does not merge them; for the small
  // workgroups of the decode kernel the count stays a constant, which keeps the kernel at five waves per SIMD)
  block_merge<(T / 64)>(st, s_m, s_l, s_acc, T > 256 ? min(T / 64, (row_b - row_a + 15) / 16) : T / 64, M, L, o);

  if (n_active == 1) {  // the only split of this head: finish here
    if (tid < kHeadDim) {
      store_out(a.out, a.out_is_bf16, head, tid, o / L);
      if (a.lse && tid == 0) a.lse[head] = (M + log2f(L)) * kLn2;
    }
    return;
  }

  // Partials are exchanged through device-coherent (agent-scope) stores and loads, which go
  // straight to memory: no L2 write-back or invalidate of the whole cache is needed around the
  // arrival counter, only "my stores have completed" before the ticket is taken.  (This leans on
  // how gfx950 handles such accesses -- they are performed at the memory side in issue order once
  // s_waitcnt has seen them complete -- rather than on release / acquire fences, which here write
  // back and invalidate the whole L2 and made the kernel four times slower.)
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

// The queue of one launch.  kCoherent = the plan was written by workgroups of this same launch: it is read with
// device-coherent loads and EVERY item is claimed from the counter (a workgroup may be missing from the launch's
// tail, see the selection kernel); otherwise a workgroup's first item is its block index and only further items
// are claimed.  Call with the whole workgroup.
template <int T, bool kGathered, bool kCoherent>
__device__ __forceinline__ void decode_queue(const DecodeArgs &a, int *s_start, int *s_src, float *s_m, float *s_l,
                                             float (*s_acc)[kHeadDim], int *s_last, int *s_item, int *s_first,
                                             int *s_scan, int *s_rows) {
  const int tid = threadIdx.x, lane16 = tid & 15, grp = tid >> 4;

  // ---- the queue: items per head from head_rows[], exclusive prefix in LDS ----
  constexpr int kMinItemChunks = T / 64;  // least chunks per item of a heavy launch: four steps of a small workgroup, two of a large one
  constexpr int kPer = kMaxQueueHeads / T;  // consecutive heads per thread
  int rows[kPer], chunks = 0;
#pragma unroll
  for (int u = 0; u < kPer; ++u) {
    const int hh = tid * kPer + u;
    // (an unconditional load at a clamped index, the value chosen afterwards: loads inside a condition are waited
    // for one by one, four dependent round trips at the start of every workgroup)
    // (Only in the decode launch of its own: inside the selection's launch the same rewrite changed nothing for the
    // queue and cost the selection of a peaked head 0.2 us through the code around it.)
    if (!kCoherent) {
      const int got = a.plan.head_rows[a.head0 + min(hh, a.n_heads - 1)];
      rows[u] = hh < a.n_heads ? got : 0;  // <= 0: nothing to do (empty, or attended already)
    } else {
      rows[u] = hh < a.n_heads ? DP_LD_I32(a.plan.head_rows[a.head0 + hh]) : 0;
    }
    s_rows[hh] = rows[u];
    if (rows[u] > 0) chunks += min(1 << 20, (rows[u] + kChunkRows - 1) / kChunkRows);  // capped: the sum stays in range
  }
  // least chunks per item, between 1 and kMinItemChunks.  A launch of many small workgroups aims at about one item
  // for every second workgroup; the few large workgroups of a shared launch (kCoherent) at four items each, in whole
  // steps of the workgroup (T / 4 rows).
  const int all_chunks = block_sum<int, (T / 64)>(chunks, s_scan);
  int g;
  if (kCoherent) {
    constexpr int kStepRows = T / 16 * queue_batch(true);
    constexpr int kStepChunks = kStepRows >= kChunkRows ? kStepRows / kChunkRows : 1;
    const int want = max(1, 4 * (int)gridDim.x);
    g = (all_chunks + want - 1) / want;
    g = min(kMinItemChunks, max(kStepChunks, (g + kStepChunks - 1) / kStepChunks * kStepChunks));
  } else {
    const int half_grid = max(1, (int)gridDim.x / 2);
    g = min(kMinItemChunks, max(1, (all_chunks + half_grid - 1) / half_grid));
  }
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
  int run = block_excl_scan<int, (T / 64)>(mine, s_scan, total);
#pragma unroll
  for (int u = 0; u < kPer; ++u) {
    s_first[tid * kPer + u] = run;
    run += cnt[u];
  }
  if (tid == T - 1) s_first[kMaxQueueHeads] = total;
  __syncthreads();
  if (total == 0) return;

  if (kCoherent) {
    // every item is claimed from the counter, the next one before this one is attended (the counter's round trip
    // hides behind the rows of a large workgroup's item)
    if (tid == 0) *s_item = __hip_atomic_fetch_add(a.queue_next, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    int item = *s_item;
    __syncthreads();
#pragma unroll 1
    while (item < total) {
      int lo = 0, hi = kMaxQueueHeads;
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (s_first[mid] <= item) lo = mid; else hi = mid;
      }
      const int head = a.head0 + lo, split = item - s_first[lo];
      int next = total;
      if (tid == 0) next = __hip_atomic_fetch_add(a.queue_next, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      decode_item<T, kGathered, true>(a, head, split, s_rows[lo], g, s_start, s_src, s_m, s_l, s_acc, s_last, tid, lane16, grp);
      if (tid == 0) *s_item = next;
      __syncthreads();  // also: LDS is reused by the next item
      item = *s_item;
      __syncthreads();
    }
    return;
  }
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
    decode_item<T, kGathered, false>(a, head, split, s_rows[lo], g, s_start, s_src, s_m, s_l, s_acc, s_last, tid, lane16, grp);
    if (total <= (int)gridDim.x) break;  // every item had its workgroup: nothing to claim
    if (tid == 0)
      *s_item = gridDim.x + __hip_atomic_fetch_add(a.queue_next, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();  // also: LDS is reused by the next item
    item = *s_item;
    __syncthreads();
  }
}

}  // namespace dp
