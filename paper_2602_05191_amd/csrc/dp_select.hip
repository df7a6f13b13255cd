// Stage 2: per-head softmax over cluster logits (paper Eq. 6), first top-p
// (Eq. 7) and second top-p (Sec. 4.3), without sorting.
//
// The retained set is a prefix of the order (logit descending, cluster index
// ascending), so it is fully described by its LAST element (key*, idx*):
//   i is retained  <=>  key_i > key*  or  (key_i == key* and i <= idx*).
// One workgroup of 1024 threads per head finds that element by threshold
// search on cumulative mass:
//   1. block max; weights w_i = exp(l_i - max) are converted to 2^-40 fixed
//      point (u64), so every sum below is an integer sum: associative, hence
//      independent of atomics order and bitwise reproducible;
//   2. an LDS histogram of mass over 2048 bins that are linear in (max - l_i)
//      (monotone in the logit), then a block scan locates the bin in which the
//      cumulative mass crosses the target;
//   3. inside that bin: if it holds few clusters, rank them exactly (pairwise
//      comparison on (key, index)); otherwise split the bin's key range into
//      2048 sub-ranges and repeat; a bin that holds one distinct key is a run
//      of ties and is cut in cluster-index order.
// The second threshold reuses the level-1 histogram.  Finally the two sets are
// compacted in ascending cluster index with block scans, together with the
// row-prefix plan that stage 3 uses to split work.
//
// Each thread keeps E consecutive logits in registers (E * 1024 >= clusters).
#include <limits.h>

#include "dp_device.hpp"
#include "dp_kernels.hpp"

namespace dp {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kBins = 2048;            // = 2 bins per thread in the histogram scan
constexpr float kBinRange = 27.0f;     // logits further than this below the max share the last bin
constexpr int kMaxCand = 512;          // largest bin population that is ranked pairwise
constexpr float kFxOne = 1099511627776.0f;  // 2^40

typedef unsigned long long u64;

struct SelectArgs {
  const float *logits;
  const int32_t *seg_cluster_ptr, *cluster_sizes, *cluster_offsets;
  int32_t n_kv_heads, n_q_heads, group, max_k;
  float p1, p2;
  uint32_t p2_absolute;
  SelectOut out;
  Plan plan;
};

__device__ __forceinline__ u64 fx_mass(float l, float mx) {
  if (l == -INFINITY) return 0;
  return (u64)(expf(l - mx) * kFxOne);
}

__device__ __forceinline__ int level1_bin(float l, float mx) {
  const float t = (mx - l) * ((float)(kBins - 1) / kBinRange);
  return t >= (float)(kBins - 1) ? kBins - 1 : (int)t;  // also catches +inf
}

struct Shared {
  u64 hist[kBins];
  u64 hist2[kBins];
  u64 scr64[kSelWaves + 1];
  float scrf[kSelWaves + 1];
  int scri[kSelWaves + 1];
  uint32_t red_lo[kSelWaves], red_hi[kSelWaves];
  int red_cnt[kSelWaves];
  uint32_t cand_key[kMaxCand];
  int cand_idx[kMaxCand];
  u64 cand_m[kMaxCand];
  int ncand;
  int bin;
  u64 before;
  uint32_t res_key;
  int res_idx;
  u64 res_mass;
};

// locate the bin of `h` in which the running sum reaches tau; 2 bins per thread
__device__ __forceinline__ void locate_bin(const u64 *h, u64 tau, Shared &sh) {
  const int t = threadIdx.x;
  const u64 h0 = h[2 * t], h1 = h[2 * t + 1];
  u64 tot;
  const u64 ex = block_excl_scan<u64, kSelWaves>(h0 + h1, sh.scr64, tot);
  if (ex < tau && tau <= ex + h0) {
    sh.bin = 2 * t;
    sh.before = ex;
  } else if (ex + h0 < tau && tau <= ex + h0 + h1) {
    sh.bin = 2 * t + 1;
    sh.before = ex + h0;
  }
  __syncthreads();
}

// count / min key / max key of the calling threads' members
__device__ __forceinline__ void reduce_members(int cnt, uint32_t lo, uint32_t hi, Shared &sh, int &cnt_o,
                                               uint32_t &lo_o, uint32_t &hi_o) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    cnt += __shfl_xor(cnt, d, 64);
    lo = min(lo, (uint32_t)__shfl_xor((int)lo, d, 64));
    hi = max(hi, (uint32_t)__shfl_xor((int)hi, d, 64));
  }
  if (lane_id() == 0) {
    sh.red_cnt[wave_id()] = cnt;
    sh.red_lo[wave_id()] = lo;
    sh.red_hi[wave_id()] = hi;
  }
  __syncthreads();
  int c = 0;
  uint32_t l = 0xffffffffu, h = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    c += sh.red_cnt[w];
    l = min(l, sh.red_lo[w]);
    h = max(h, sh.red_hi[w]);
  }
  __syncthreads();
  cnt_o = c;
  lo_o = l;
  hi_o = h;
}

// Last element (key, index) of the shortest prefix of the order whose mass
// reaches tau, and that prefix's mass.  Requires 1 <= tau <= total mass and a
// level-1 histogram in sh.hist.  Block-uniform control flow throughout.
template <int E>
__device__ __forceinline__ void find_prefix(const float (&l)[E], float mx, int base, u64 tau, Shared &sh,
                                            uint32_t &key_o, int &idx_o, u64 &mass_o) {
  const int tid = threadIdx.x;
  locate_bin(sh.hist, tau, sh);
  const int bin1 = sh.bin;
  u64 before = sh.before;

  // members of the crossing bin: count and key range.  The bins are monotone
  // in the logit, so from here on "member" means  klo <= key <= khi.
  int cnt;
  uint32_t klo, khi;
  {
    int c = 0;
    uint32_t lo = 0xffffffffu, hi = 0;
#pragma unroll
    for (int e = 0; e < E; ++e)
      if (l[e] != -INFINITY && level1_bin(l[e], mx) == bin1) {
        const uint32_t k = ordered_key(l[e]);
        ++c;
        lo = min(lo, k);
        hi = max(hi, k);
      }
    reduce_members(c, lo, hi, sh, cnt, klo, khi);
  }

  // split the key range until the members can be ranked or are all ties
#pragma unroll 1
  while (cnt > kMaxCand && klo != khi) {
    for (int i = tid; i < kBins; i += kSelThreads) sh.hist2[i] = 0;
    __syncthreads();
    const u64 span = (u64)(khi - klo) + 1;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const uint32_t k = ordered_key(l[e]);
      if (l[e] != -INFINITY && k >= klo && k <= khi) {
        const u64 m = fx_mass(l[e], mx);
        if (m) atomicAdd(&sh.hist2[(int)(((u64)(khi - k) * kBins) / span)], m);
      }
    }
    __syncthreads();
    locate_bin(sh.hist2, tau - before, sh);
    const int bin2 = sh.bin;
    before += sh.before;
    int c = 0;
    uint32_t lo = 0xffffffffu, hi = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const uint32_t k = ordered_key(l[e]);
      if (l[e] != -INFINITY && k >= klo && k <= khi && (int)(((u64)(khi - k) * kBins) / span) == bin2) {
        ++c;
        lo = min(lo, k);
        hi = max(hi, k);
      }
    }
    reduce_members(c, lo, hi, sh, cnt, klo, khi);
  }

  if (cnt <= kMaxCand) {
    // rank the members exactly on (key descending, index ascending)
    if (tid == 0) sh.ncand = 0;
    __syncthreads();
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const uint32_t k = ordered_key(l[e]);
      if (l[e] != -INFINITY && k >= klo && k <= khi) {
        const int slot = atomicAdd(&sh.ncand, 1);
        sh.cand_key[slot] = k;
        sh.cand_idx[slot] = base + e;
        sh.cand_m[slot] = fx_mass(l[e], mx);
      }
    }
    __syncthreads();
    if (tid < cnt) {
      const uint32_t ki = sh.cand_key[tid];
      const int ii = sh.cand_idx[tid];
      const u64 mi = sh.cand_m[tid];
      u64 ahead = before;
      for (int j = 0; j < cnt; ++j) {
        const uint32_t kj = sh.cand_key[j];
        if (kj > ki || (kj == ki && sh.cand_idx[j] < ii)) ahead += sh.cand_m[j];
      }
      if (ahead < tau && tau <= ahead + mi) {  // true for exactly one member
        sh.res_key = ki;
        sh.res_idx = ii;
        sh.res_mass = ahead + mi;
      }
    }
    __syncthreads();
  } else {
    // one distinct key: a run of ties of equal mass, cut in cluster-index order
    int c = 0;
    u64 mm = 0;
#pragma unroll
    for (int e = 0; e < E; ++e)
      if (l[e] != -INFINITY && ordered_key(l[e]) == klo) {
        ++c;
        mm = fx_mass(l[e], mx);
      }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
      const u64 o = __shfl_xor(mm, d, 64);
      mm = o > mm ? o : mm;
    }
    if (lane_id() == 0) sh.scr64[wave_id()] = mm;
    __syncthreads();
    u64 m_tie = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) m_tie = sh.scr64[w] > m_tie ? sh.scr64[w] : m_tie;
    __syncthreads();
    const u64 need = (tau - before + m_tie - 1) / m_tie;  // ties taken, 1 <= need <= cnt
    int tot;
    const int ex = block_excl_scan<int, kSelWaves>(c, sh.scri, tot);
    if ((u64)ex < need && need <= (u64)(ex + c)) {
      int seen = ex;
#pragma unroll
      for (int e = 0; e < E; ++e)
        if (l[e] != -INFINITY && ordered_key(l[e]) == klo) {
          ++seen;
          if ((u64)seen == need) {
            sh.res_key = klo;
            sh.res_idx = base + e;
            sh.res_mass = before + need * m_tie;
          }
        }
    }
    __syncthreads();
  }
  key_o = sh.res_key;
  idx_o = sh.res_idx;
  mass_o = sh.res_mass;
  __syncthreads();  // sh.res_* / sh.bin may be rewritten by the next search
}

template <int E>
__global__ __launch_bounds__(kSelThreads) void select_kernel(SelectArgs a) {
  __shared__ Shared sh;
  const int head = blockIdx.x;
  const int b = head / a.n_q_heads, h = head % a.n_q_heads;
  const int seg = b * a.n_kv_heads + h / a.group;
  const int c0 = a.seg_cluster_ptr[seg];
  const int kc = a.seg_cluster_ptr[seg + 1] - c0;
  const float *lg = a.logits + (int64_t)a.group * c0 + (int64_t)(h % a.group) * kc;
  const int tid = threadIdx.x;
  const int base = tid * E;

  int32_t *sel = a.out.sel_ids + (int64_t)head * a.max_k;
  const bool plan = a.plan.ent_src != nullptr;
  int32_t *ent_src = plan ? a.plan.ent_src + (int64_t)head * a.max_k : nullptr;
  int32_t *row_start = plan ? a.plan.row_start + (int64_t)head * (a.max_k + 1) : nullptr;
  int32_t *chunk_entry = plan ? a.plan.chunk_entry + (int64_t)head * a.plan.chunk_stride : nullptr;

  // ---- load, max ---------------------------------------------------------
  float l[E];
  float tmax = -INFINITY;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int i = base + e;
    l[e] = (i < kc) ? lg[i] + 0.0f : -INFINITY;  // +0.0f: -0 becomes +0
    tmax = fmaxf(tmax, l[e]);
  }
  for (int i = tid; i < kBins; i += kSelThreads) sh.hist[i] = 0;
  const float mx = block_max<kSelWaves>(tmax, sh.scrf);  // barriers also publish the zeroed histogram

  if (mx == -INFINITY) {  // no non-empty cluster
    if (tid == 0) {
      a.out.n_exact[head] = 0;
      a.out.n_retained[head] = 0;
      a.out.n_exact_tokens[head] = 0;
      if (plan) {
        row_start[0] = 0;
        a.plan.head_rows[head] = 0;
      }
    }
    return;
  }

  // ---- level-1 mass histogram and total mass -----------------------------
  u64 wsum = 0;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const u64 m = fx_mass(l[e], mx);
    if (m) {
      atomicAdd(&sh.hist[level1_bin(l[e], mx)], m);
      wsum += m;
    }
  }
  const u64 W = block_sum<u64, kSelWaves>(wsum, sh.scr64);  // >= 2^40: the max element has weight 1

  // ---- the two thresholds -------------------------------------------------
  uint32_t key1, key2;
  int idx1, idx2;
  u64 mass1;
  if (a.p1 >= 1.0f) {  // every non-empty cluster
    key1 = kKeyLowestFinite;
    idx1 = INT_MAX;
    mass1 = W;
  } else {
    u64 tau = (u64)ceil((double)a.p1 * (double)W);
    tau = tau < 1 ? 1 : (tau > W ? W : tau);
    find_prefix<E>(l, mx, base, tau, sh, key1, idx1, mass1);
  }
  if (a.p2 >= 1.0f) {
    key2 = key1;
    idx2 = idx1;
  } else if (a.p2 <= 0.0f) {  // nothing is exact
    key2 = 0xffffffffu;
    idx2 = -1;
  } else {
    u64 tau = a.p2_absolute ? (u64)ceil((double)a.p2 * (double)W) : (u64)ceil((double)a.p2 * (double)mass1);
    tau = tau < 1 ? 1 : (tau > mass1 ? mass1 : tau);
    u64 mass2;
    find_prefix<E>(l, mx, base, tau, sh, key2, idx2, mass2);
  }

  // ---- compaction in ascending cluster index ------------------------------
  int ce = 0, ca = 0, te = 0;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    if (l[e] == -INFINITY) continue;
    const uint32_t k = ordered_key(l[e]);
    const int i = base + e;
    const bool ret = k > key1 || (k == key1 && i <= idx1);
    const bool exa = k > key2 || (k == key2 && i <= idx2);
    if (exa) {
      ++ce;
      te += a.cluster_sizes[c0 + i];
    } else if (ret) {
      ++ca;
    }
  }
  int n_ex, n_ap, n_tok;
  int pe = block_excl_scan<int, kSelWaves>(ce, sh.scri, n_ex);
  int pa = block_excl_scan<int, kSelWaves>(ca, sh.scri, n_ap);
  int pt = block_excl_scan<int, kSelWaves>(te, sh.scri, n_tok);
#pragma unroll
  for (int e = 0; e < E; ++e) {
    if (l[e] == -INFINITY) continue;
    const uint32_t k = ordered_key(l[e]);
    const int i = base + e;
    const bool ret = k > key1 || (k == key1 && i <= idx1);
    const bool exa = k > key2 || (k == key2 && i <= idx2);
    if (exa) {
      sel[pe] = i;
      const int sz = a.cluster_sizes[c0 + i];
      if (plan) {
        ent_src[pe] = a.cluster_offsets[c0 + i];
        row_start[pe] = pt;
        for (int q = (pt + kChunkRows - 1) / kChunkRows; q * kChunkRows < pt + sz; ++q) chunk_entry[q] = pe;
      }
      ++pe;
      pt += sz;
    } else if (ret) {
      const int j = n_ex + pa;
      sel[j] = i;
      if (plan) {
        const int row = n_tok + pa;
        ent_src[j] = i;
        row_start[j] = row;
        if (row % kChunkRows == 0) chunk_entry[row / kChunkRows] = j;
      }
      ++pa;
    }
  }
  if (tid == 0) {
    a.out.n_exact[head] = n_ex;
    a.out.n_retained[head] = n_ex + n_ap;
    a.out.n_exact_tokens[head] = n_tok;
    if (plan) {
      row_start[n_ex + n_ap] = n_tok + n_ap;
      a.plan.head_rows[head] = n_tok + n_ap;
    }
  }
}

// ---- plan from caller-given sets (staged API) -----------------------------
constexpr int kPlanThreads = 256;

struct PlanArgs {
  const int32_t *seg_cluster_ptr, *cluster_sizes, *cluster_offsets;
  const int32_t *sel_ids, *n_exact, *n_retained;
  int32_t *n_exact_tokens;  // nullable
  int32_t n_kv_heads, n_q_heads, group, max_k;
  Plan plan;
};

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(PlanArgs a) {
  __shared__ int scr[kPlanThreads / 64 + 1];
  const int head = blockIdx.x;
  const int b = head / a.n_q_heads, h = head % a.n_q_heads;
  const int seg = b * a.n_kv_heads + h / a.group;
  const int c0 = a.seg_cluster_ptr[seg];
  const int n_ex = a.n_exact[head], n_rt = a.n_retained[head];
  const int32_t *sel = a.sel_ids + (int64_t)head * a.max_k;
  int32_t *ent_src = a.plan.ent_src + (int64_t)head * a.max_k;
  int32_t *row_start = a.plan.row_start + (int64_t)head * (a.max_k + 1);
  int32_t *chunk_entry = a.plan.chunk_entry + (int64_t)head * a.plan.chunk_stride;
  const int tid = threadIdx.x;

  int carry = 0;
  for (int j0 = 0; j0 < n_ex; j0 += kPlanThreads) {
    const int j = j0 + tid;
    int id = 0, sz = 0;
    if (j < n_ex) {
      id = sel[j];
      sz = a.cluster_sizes[c0 + id];
    }
    int tot;
    const int pt = carry + block_excl_scan<int, kPlanThreads / 64>(sz, scr, tot);
    if (j < n_ex) {
      ent_src[j] = a.cluster_offsets[c0 + id];
      row_start[j] = pt;
      for (int q = (pt + kChunkRows - 1) / kChunkRows; q * kChunkRows < pt + sz; ++q) chunk_entry[q] = j;
    }
    carry += tot;
  }
  const int n_tok = carry;
  for (int j = n_ex + tid; j < n_rt; j += kPlanThreads) {
    const int row = n_tok + (j - n_ex);
    ent_src[j] = sel[j];
    row_start[j] = row;
    if (row % kChunkRows == 0) chunk_entry[row / kChunkRows] = j;
  }
  if (tid == 0) {
    row_start[n_rt] = n_tok + (n_rt - n_ex);
    a.plan.head_rows[head] = n_tok + (n_rt - n_ex);
    if (a.n_exact_tokens) a.n_exact_tokens[head] = n_tok;
  }
}

}  // namespace

hipError_t launch_select(const CacheView &c, const float *logits, float p1, float p2, uint32_t flags,
                         const SelectOut &out, const Plan &plan, hipStream_t s) {
  SelectArgs a;
  a.logits = logits;
  a.seg_cluster_ptr = c.seg_cluster_ptr;
  a.cluster_sizes = c.cluster_sizes;
  a.cluster_offsets = c.cluster_offsets;
  a.n_kv_heads = c.n_kv_heads;
  a.n_q_heads = c.n_q_heads;
  a.group = c.group;
  a.max_k = c.max_clusters_per_seg;
  a.p1 = p1;
  a.p2 = p2;
  a.p2_absolute = flags & 1u;
  a.out = out;
  a.plan = plan;
  const dim3 grid(c.batch * c.n_q_heads), block(kSelThreads);
  if (grid.x == 0) return hipSuccess;
  const int k = c.max_clusters_per_seg;
  if (k <= 2 * kSelThreads) hipLaunchKernelGGL(select_kernel<2>, grid, block, 0, s, a);
  else if (k <= 4 * kSelThreads) hipLaunchKernelGGL(select_kernel<4>, grid, block, 0, s, a);
  else if (k <= 8 * kSelThreads) hipLaunchKernelGGL(select_kernel<8>, grid, block, 0, s, a);
  else if (k <= 16 * kSelThreads) hipLaunchKernelGGL(select_kernel<16>, grid, block, 0, s, a);
  else if (k <= 32 * kSelThreads) hipLaunchKernelGGL(select_kernel<32>, grid, block, 0, s, a);
  else if (k <= 64 * kSelThreads) hipLaunchKernelGGL(select_kernel<64>, grid, block, 0, s, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_plan(const CacheView &c, const int32_t *sel_ids, const int32_t *n_exact,
                       const int32_t *n_retained, int32_t *n_exact_tokens, const Plan &plan, hipStream_t s) {
  PlanArgs a;
  a.seg_cluster_ptr = c.seg_cluster_ptr;
  a.cluster_sizes = c.cluster_sizes;
  a.cluster_offsets = c.cluster_offsets;
  a.sel_ids = sel_ids;
  a.n_exact = n_exact;
  a.n_retained = n_retained;
  a.n_exact_tokens = n_exact_tokens;
  a.n_kv_heads = c.n_kv_heads;
  a.n_q_heads = c.n_q_heads;
  a.group = c.group;
  a.max_k = c.max_clusters_per_seg;
  a.plan = plan;
  const dim3 grid(c.batch * c.n_q_heads);
  if (grid.x == 0) return hipSuccess;
  hipLaunchKernelGGL(plan_kernel, grid, dim3(kPlanThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace dp
