// A/B variants that follow the kernel structure the paper describes for its own
// implementation (Sec. 4.4), kept next to the product kernels so that the two
// designs can be timed against each other on the same inputs.  They compute the
// same results (same order, same fixed-point masses, same tie-break); nothing
// in the product path calls them.
//
//   select_sorted_kernel   "top-p on sorted tensors": sort the cluster scores of
//                          a head (bitonic sort of (score, index) keys in LDS),
//                          prefix-sum the masses along the sorted order, and cut
//                          both prefixes where the running mass reaches the threshold
//   gather_rows_kernel     "fused gathering into a contiguous buffer": the K / V
//                          rows of a head's exact clusters are copied into a
//                          per-head buffer; the decode kernel then reads that
//                          buffer instead of the cache
#include "dp_attend.hpp"
#include "dp_device.hpp"
#include "dp_kernels.hpp"
#include "dp_mass.hpp"

namespace dp {
namespace {

constexpr int kSortThreads = 1024;
constexpr int kSortWaves = kSortThreads / 64;
constexpr int kSortMax = 8192;            // clusters per segment this variant handles (64 KB of keys in LDS)
constexpr int kSortPer = kSortMax / kSortThreads;

struct SortedArgs {
  const float *logits;
  const int32_t *seg_cluster_ptr, *cluster_sizes;
  int32_t n_kv_heads, n_q_heads, group, max_k;
  float p1, p2;
  uint32_t p2_absolute;
  SelectOut out;
};

__global__ __launch_bounds__(kSortThreads) void select_sorted_kernel(SortedArgs a) {
  __shared__ u64 s_key[kSortMax];          // (ordered score key << 32) | ~index : descending = score desc, index asc
  __shared__ uint8_t s_flag[kSortMax];     // by cluster id: 2 exact, 1 approximated, 0 not selected
  __shared__ u64 scr64[kSortWaves + 1];
  __shared__ int scri[2 * (kSortWaves + 1)];
  const int head = blockIdx.x, tid = threadIdx.x;
  const int b = head / a.n_q_heads, h = head % a.n_q_heads;
  const int seg = b * a.n_kv_heads + h / a.group;
  const int c0 = a.seg_cluster_ptr[seg], kc = a.seg_cluster_ptr[seg + 1] - c0;
  const float *lg = a.logits + (int64_t)a.group * c0 + (int64_t)(h % a.group) * kc;
  int n2 = 1;
  while (n2 < kc) n2 <<= 1;                // padded length of the sort

  // ---- keys; padding and empty clusters sort to the end ----
  for (int i = tid; i < n2; i += kSortThreads) {
    const float l = i < kc ? lg[i] + 0.0f : -INFINITY;
    s_key[i] = ((u64)ordered_key(l) << 32) | (uint32_t)~(uint32_t)i;
    if (i < kSortMax) s_flag[i] = 0;
  }
  __syncthreads();
  // ---- bitonic sort, descending ----
  for (int k = 2; k <= n2; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int t = tid; t < (n2 >> 1); t += kSortThreads) {
        const int lo = ((t & ~(j - 1)) << 1) | (t & (j - 1)), hi = lo | j;  // the pair (lo, lo + j)
        const bool desc = (lo & k) == 0;
        const u64 x = s_key[lo], y = s_key[hi];
        if ((x < y) == desc) {
          s_key[lo] = y;
          s_key[hi] = x;
        }
      }
      __syncthreads();
    }
  }
  // ---- masses along the sorted order, inclusive prefix sum ----
  const uint32_t top = (uint32_t)(s_key[0] >> 32);
  const bool none = top < kKeyLowestFinite;  // every cluster is empty
  // the max logit from its key (the inverse of ordered_key)
  const float mx = __uint_as_float((top & 0x80000000u) ? (top & 0x7fffffffu) : ~top);
  u64 m[kSortPer], run = 0;
  int live = 0;                              // non-empty clusters among this thread's positions
#pragma unroll
  for (int e = 0; e < kSortPer; ++e) {
    const int i = tid * kSortPer + e;
    m[e] = 0;
    if (i < n2 && !none) {
      const uint32_t key = (uint32_t)(s_key[i] >> 32);
      if (key >= kKeyLowestFinite) {
        const float l = __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
        m[e] = fx_mass(mx - l);
        ++live;
      }
    }
    run += m[e];
  }
  u64 W;
  const u64 before = block_excl_scan<u64, kSortWaves>(run, scr64, W);
  int n_live;
  block_excl_scan<int, kSortWaves>(live, scri, n_live);

  // ---- both cuts: position i is retained iff the mass strictly before it is below the threshold ----
  int k1 = 0, k2 = 0;
  if (!none) {
    const bool all = a.p1 >= 1.0f;
    const u64 tau1 = top_p_first_tau(a.p1, W);
    // m1 = inclusive mass at the last retained position: every thread derives it from a block reduction
    u64 cum = before;
    int c1 = 0;
    u64 m1_local = 0;
#pragma unroll
    for (int e = 0; e < kSortPer; ++e) {
      if (m[e] && cum < tau1) {
        ++c1;
        m1_local = cum + m[e];
      }
      cum += m[e];
    }
    int tot1;
    block_excl_scan<int, kSortWaves>(c1, scri, tot1);
    // the retained masses are increasing along the order: the block maximum is the last one
    u64 mm = m1_local;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
      const u64 o = __shfl_xor(mm, d, 64);
      mm = o > mm ? o : mm;
    }
    if (lane_id() == 0) scr64[wave_id()] = mm;
    __syncthreads();
    u64 m1 = 0;
#pragma unroll
    for (int w = 0; w < kSortWaves; ++w) m1 = scr64[w] > m1 ? scr64[w] : m1;
    __syncthreads();
    k1 = all ? n_live : tot1;
    if (all) m1 = W;
    u64 tau2 = 0;
    const int kind = top_p_second_tau(a.p2, a.p2_absolute != 0, W, m1, tau2);
    if (kind == 1) {
      k2 = k1;
    } else if (kind == 2) {
      cum = before;
      int c2 = 0;
#pragma unroll
      for (int e = 0; e < kSortPer; ++e) {
        if (m[e] && cum < tau2) ++c2;
        cum += m[e];
      }
      block_excl_scan<int, kSortWaves>(c2, scri, k2);
    }
  }
  // ---- mark the selected clusters by id, then compact in ascending id ----
  for (int i = tid; i < k1; i += kSortThreads) s_flag[~(uint32_t)s_key[i]] = i < k2 ? 2 : 1;
  __syncthreads();
  int ce = 0, ca = 0, te = 0;
#pragma unroll
  for (int e = 0; e < kSortPer; ++e) {
    const int i = tid * kSortPer + e;
    if (i < kc) {
      ce += s_flag[i] == 2;
      ca += s_flag[i] == 1;
      if (s_flag[i] == 2) te += a.cluster_sizes[c0 + i];
    }
  }
  int n_ex, n_ap, n_tok;
  int pe = block_excl_scan<int, kSortWaves>(ce, scri, n_ex);
  int pa = block_excl_scan<int, kSortWaves>(ca, scri, n_ap);
  block_excl_scan<int, kSortWaves>(te, scri, n_tok);
  int32_t *sel = a.out.sel_ids + (int64_t)head * a.max_k;
#pragma unroll
  for (int e = 0; e < kSortPer; ++e) {
    const int i = tid * kSortPer + e;
    if (i < kc) {
      if (s_flag[i] == 2) sel[pe++] = i;
      else if (s_flag[i] == 1) sel[n_ex + pa++] = i;
    }
  }
  if (tid == 0) {
    a.out.n_exact[head] = n_ex;
    a.out.n_retained[head] = n_ex + n_ap;
    a.out.n_exact_tokens[head] = n_tok;
  }
}

// ---- gather of the exact clusters' rows into a per-head contiguous buffer ----
struct GatherArgs {
  const void *k_cache, *v_cache;
  const int64_t *seg_row_base;
  const int32_t *n_exact;
  Plan plan;
  void *k_buf, *v_buf;  // [nh, rows_cap, 128] bf16
  int32_t n_kv_heads, n_q_heads, group, max_k, rows_cap;
};

__global__ __launch_bounds__(256) void gather_rows_kernel(GatherArgs a) {
  const int head = blockIdx.y;
  const int b = head / a.n_q_heads, h = head % a.n_q_heads;
  const int seg = b * a.n_kv_heads + h / a.group;
  const int n_ex = a.n_exact[head];
  const int32_t *ent_src = a.plan.ent_src + (int64_t)head * a.max_k;
  const int32_t *row_start = a.plan.row_start + (int64_t)head * (a.max_k + 1);
  const int rows = n_ex > 0 ? row_start[n_ex] : 0;  // exact rows come first in the list
  if (rows > a.rows_cap) return;  // does not fit: the decode kernel reads this head in place
  const int r0 = blockIdx.x * kChunkRows;
  if (r0 >= rows) return;
  const int lane16 = threadIdx.x & 15, grp = threadIdx.x >> 4;
  int ent = a.plan.chunk_entry[(int64_t)head * a.plan.chunk_stride + blockIdx.x];
  const int64_t src0 = a.seg_row_base[seg];
  // 16 DPP rows x 4 rows each = the chunk's 64 rows
  for (int u = 0; u < kChunkRows / 16; ++u) {
    const int row = r0 + u * 16 + grp;
    if (row >= rows) break;
    while (row >= row_start[ent + 1]) ++ent;
    const int64_t g = src0 + ent_src[ent] + (row - row_start[ent]);
    const int64_t d = (int64_t)head * a.rows_cap + row;
    *reinterpret_cast<uint4 *>(static_cast<char *>(a.k_buf) + d * kRowBytes + lane16 * 16) =
        load_row_slice(a.k_cache, g, lane16);
    *reinterpret_cast<uint4 *>(static_cast<char *>(a.v_buf) + d * kRowBytes + lane16 * 16) =
        load_row_slice(a.v_cache, g, lane16);
  }
}

}  // namespace

hipError_t launch_select_sorted(const CacheView &c, const float *logits, const SelectRule &rule, const SelectOut &out,
                                hipStream_t s) {
  const dim3 grid(c.batch * c.n_q_heads);
  if (grid.x == 0) return hipSuccess;
  if (c.max_clusters_per_seg > kSortMax) return hipErrorInvalidValue;
  SortedArgs a;
  a.logits = logits;
  a.seg_cluster_ptr = c.seg_cluster_ptr;
  a.cluster_sizes = c.cluster_sizes;
  a.n_kv_heads = c.n_kv_heads;
  a.n_q_heads = c.n_q_heads;
  a.group = c.group;
  a.max_k = c.max_clusters_per_seg;
  a.p1 = rule.p1;
  a.p2 = rule.p2;
  a.p2_absolute = rule.p2_absolute;
  a.out = out;
  hipLaunchKernelGGL(select_sorted_kernel, grid, dim3(kSortThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_gather_rows(const CacheView &c, const int32_t *n_exact, const Plan &plan, void *k_buf, void *v_buf,
                              int rows_cap, hipStream_t s) {
  const int nh = c.batch * c.n_q_heads;
  if (nh == 0 || rows_cap <= 0) return hipSuccess;
  GatherArgs a;
  a.k_cache = c.k_cache;
  a.v_cache = c.v_cache;
  a.seg_row_base = c.seg_row_base;
  a.n_exact = n_exact;
  a.plan = plan;
  a.k_buf = k_buf;
  a.v_buf = v_buf;
  a.n_kv_heads = c.n_kv_heads;
  a.n_q_heads = c.n_q_heads;
  a.group = c.group;
  a.max_k = c.max_clusters_per_seg;
  a.rows_cap = rows_cap;
  hipLaunchKernelGGL(gather_rows_kernel, dim3((rows_cap + kChunkRows - 1) / kChunkRows, nh), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace dp
