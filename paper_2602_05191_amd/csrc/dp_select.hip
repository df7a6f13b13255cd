// Stage 2: per-head softmax over cluster logits (paper Eq. 6), first top-p
// (Eq. 7) and second top-p (Sec. 4.3), without sorting.
//
// The retained set is a prefix of the order (logit descending, cluster index
// ascending), so it is fully described by its LAST element (key*, idx*):
//   i is retained  <=>  key_i > key*  or  (key_i == key* and i <= idx*).
// One workgroup of 1024 threads per head finds that element by threshold
// search on cumulative mass; each thread keeps E consecutive logits in
// registers (E * 1024 >= clusters of the segment).
//   1. block max.  Weights w_i = exp(l_i - max) are converted to 2^-40 fixed
//      point (u64), so every sum below is an integer sum: associative, hence
//      independent of the order of the LDS atomics and bitwise reproducible.
//      A logit more than 40 ln 2 below the max has mass 0 and is out of play.
//   2. an LDS histogram of mass over 2048 bins that are linear in (max - l_i)
//      (monotone in the logit); one block scan gives the total mass and, for
//      both thresholds, the bin in which the cumulative mass crosses it.
//   3. inside that bin: if it holds at most 512 clusters (the normal case: a
//      handful), rank them exactly by pairwise comparison on (key, index);
//      otherwise split the bin's key range into 2048 sub-ranges and repeat; a
//      bin that holds one distinct key is a run of ties, cut in index order.
//   4. the two sets are compacted in ascending cluster index with one block
//      scan, together with the row-prefix plan that stage 3 splits work by.
//   Fast path (tried first): when at most 64 clusters lie within 6 of the max
//      logit and their mass already reaches the first threshold (a peaked head),
//      the retained set is inside that top set; one wave ranks it pairwise and
//      emits both lists, and steps 2-4 are skipped.  Same masses, same result.
//   5. one-call path only: a head with at most 1024 rows is attended right
//      here (64 DPP-row groups), which saves the latency of two more kernels
//      for sharply peaked heads; heavier heads go to the split decode kernel.
#include <hip/hip_ext.h>
#include <limits.h>

#include "dp_decode_body.hpp"
#include "dp_mass.hpp"

namespace dp {
namespace {

constexpr int kSelThreads = 1024;             // largest workgroup; launches with more heads than CUs use 512 or 256
constexpr int kSelWaves = kSelThreads / 64;   // the small LDS scratch arrays are sized for the largest workgroup
// level-1 histogram bins, by workgroup size T (2 or 4 consecutive bins per thread in the scan)
constexpr int bins_of(int T) { return T >= 512 ? 2048 : 1024; }
constexpr int log2_bins_of(int T) { return T >= 512 ? 11 : 10; }
// heads with at most this many rows are attended inside the selection kernel (T / 16 DPP rows, 16 rows each)
constexpr int inline_rows_of(int T) { return T; }
constexpr int kMaxCand = 512;            // largest bin population that is ranked pairwise
constexpr float kTopCut = 6.0f;          // "top set": clusters whose logit is within this of the max
constexpr int kTopMax = 64;              // largest top set handled by the one-wave fast path
// Selection from the scoring kernel's sub-tile summaries (one-call path): one wave reads them, up to this many per
// lane (8192 clusters), and the top set may spread over at most this many sub-tiles (one lane per cluster of those)
constexpr int kLiteSubPerLane = 8;
constexpr int kLiteMaxTopSub = 4;



struct SelectArgs {
  const float *logits;
  const int32_t *seg_cluster_ptr, *cluster_sizes, *cluster_offsets;
  const uint8_t *cluster_flags;  // nullable; bit 0: pinned cluster (out of the distribution, always exact)
  int32_t n_kv_heads, n_q_heads, group, max_k;
  int32_t uniform_kc;  // > 0: every segment has exactly this many clusters (no CSR lookup needed)
  const float2 *summaries;  // nullable: the scoring kernel's (max, sum exp) per head and sub-tile, row stride sub_stride
  int32_t sub_stride;
  float p1, p2;
  uint32_t p2_absolute;
  int32_t k_retained, k_exact;  // fixed-budget rule (the kernel's kCount variant): counts instead of p1, p2
  SelectOut out;
  Plan plan;
  // inline attention (one-call path); out == nullptr disables it
  const void *q, *k_cache, *v_cache, *k_centroids, *v_centroids;
  const int64_t *seg_row_base;
  void *attn_out;
  float *lse;
  int32_t out_is_bf16;
  float scale_log2;
};

// level-1 bin of a cluster at distance d below the max logit; bs = bins per unit of d
__device__ __forceinline__ int level1_bin(float d, float bs, int bins) { return (int)fminf(d * bs, (float)(bins - 1)); }

// The same threshold search serves two rules.  Top-p (kCount = false): a cluster weighs its
// fixed-point softmax mass and is in play while that mass is non-zero.  Fixed budget (kCount =
// true): every non-empty cluster weighs 1, so "the shortest prefix whose weight reaches k" is
// the top-k of the order; its level-1 bins are spread over the head's own range of logits
// (max - min), because clusters far below the max still count.
template <bool kCount>
__device__ __forceinline__ bool in_play(float d) { return kCount ? d < INFINITY : d < kCut; }
template <bool kCount>
__device__ __forceinline__ u64 mass_of(float d) { return kCount ? (u64)(d < INFINITY) : fx_mass(d); }

template <int T>
struct Shared {
  u64 hist[bins_of(T)];
  u64 scr64[kSelWaves], scr64b[kSelWaves];
  float scrf[kSelWaves];
  int scri[3 * kSelWaves];
  uint32_t red_lo[kSelWaves], red_hi[kSelWaves];
  int red_cnt[kSelWaves];
  uint32_t cand_key[kMaxCand];
  int cand_idx[kMaxCand];
  u64 cand_m[kMaxCand];
  u64 cand_ahead[kMaxCand];  // weight that precedes a candidate inside its bin, summed by slices of the block
  int ncand[2];
  int bin;
  u64 before;
  uint32_t res_key;
  int res_idx;
  u64 res_mass;
  // fast path: the top set
  uint32_t top_key[kTopMax];
  int top_idx[kTopMax], top_sz[kTopMax], top_off[kTopMax];
  u64 top_m[kTopMax];
  int ntop, f_nex, f_nap, f_ntok;
  float lite_max;                // the head's max logit as the summaries give it (exact), for the general path
  // The refinement histogram of the (rare) crowded-bin search and the lists / merge buffers of the inline
  // attention never live at the same time: the lists are written once the search is over.
  union {
    u64 hist2[bins_of(T)];
    struct {
      int l_start[inline_rows_of(T) + 1];
      int l_src[inline_rows_of(T)];
      float m_m[kSelWaves], m_l[kSelWaves];
      float m_acc[T / 64][kHeadDim];
    } at;
  };
};

// count / min key / max key over the block
template <int T>
__device__ __forceinline__ void reduce_members(int cnt, uint32_t lo, uint32_t hi, Shared<T> &sh, int &cnt_o,
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
  for (int w = 0; w < (T / 64); ++w) {
    c += sh.red_cnt[w];
    l = min(l, sh.red_lo[w]);
    h = max(h, sh.red_hi[w]);
  }
  __syncthreads();
  cnt_o = c;
  lo_o = l;
  hi_o = h;
}

// Rare path: the crossing bin holds more than kMaxCand clusters.  Narrow the key range
// [klo, khi] (by up-to-2048-way splits of the key range, re-histogrammed in sh.hist2) until the members can
// be ranked, or are a run of equal keys which is cut in index order.  On return either
// cnt <= kMaxCand (members = keys in [klo, khi], not yet gathered) or done and the result is in sh.res_*.
// The logits are read again from memory in rolled loops, so that this path adds nothing to the register
// pressure of the common one (it costs a few global round trips per pass instead).  `masked`: bit e set = this
// thread's element e carries a cluster flag and is outside the distribution, whatever its stored logit.
struct Refined {
  u64 before;
  uint32_t klo, khi;
  int cnt;
  bool done;
};
template <int E, bool kCount, int T>
__device__ __forceinline__ Refined refine_or_cut_ties(const float *lg, int kc, float mx, float bs, int base, int bin1,
                                                      u64 tau, u64 before, u64 masked, Shared<T> *shp) {
  Shared<T> &sh = *shp;
  constexpr int kBins = bins_of(T);
  const int tid = threadIdx.x;
  auto logit = [&](int e) { return (base + e < kc && !((masked >> e) & 1)) ? lg[base + e] + 0.0f : -INFINITY; };
  uint32_t klo, khi;
  int cnt;
  {
    int c = 0;
    uint32_t lo = 0xffffffffu, hi = 0;
#pragma unroll 1
    for (int e = 0; e < E; ++e) {
      const float le = logit(e), d = mx - le;
      if (in_play<kCount>(d) && level1_bin(d, bs, kBins) == bin1) {
        const uint32_t k = ordered_key(le);
        ++c;
        lo = min(lo, k);
        hi = max(hi, k);
      }
    }
    reduce_members<T>(c, lo, hi, sh, cnt, klo, khi);
  }
#pragma unroll 1
  while (cnt > kMaxCand && klo != khi) {
    for (int i = tid; i < kBins; i += T) sh.hist2[i] = 0;
    __syncthreads();
    // kBins-way split of the key range by a shift: monotone in the key, no division
    const int shift = max(0, 32 - __clz(khi - klo) - log2_bins_of(T));
#pragma unroll 1
    for (int e = 0; e < E; ++e) {
      const float le = logit(e), d = mx - le;
      const uint32_t k = ordered_key(le);
      if (in_play<kCount>(d) && k >= klo && k <= khi) {
        const u64 m = mass_of<kCount>(d);
        if (m) atomicAdd(&sh.hist2[(khi - k) >> shift], m);
      }
    }
    __syncthreads();
    {
      constexpr int B = kBins / T;  // consecutive bins per thread
      u64 hb[B], sum = 0;
#pragma unroll
      for (int q = 0; q < B; ++q) {
        hb[q] = sh.hist2[B * tid + q];
        sum += hb[q];
      }
      u64 tot;
      u64 run = block_excl_scan<u64, (T / 64)>(sum, sh.scr64, tot);
      const u64 t2 = tau - before;
#pragma unroll
      for (int q = 0; q < B; ++q) {
        if (run < t2 && t2 <= run + hb[q]) {
          sh.bin = B * tid + q;
          sh.before = run;
        }
        run += hb[q];
      }
      __syncthreads();
    }
    const int bin2 = sh.bin;
    before += sh.before;
    int c = 0;
    uint32_t lo = 0xffffffffu, hi = 0;
#pragma unroll 1
    for (int e = 0; e < E; ++e) {
      const float le = logit(e), d = mx - le;
      const uint32_t k = ordered_key(le);
      if (in_play<kCount>(d) && k >= klo && k <= khi && (int)((khi - k) >> shift) == bin2) {
        ++c;
        lo = min(lo, k);
        hi = max(hi, k);
      }
    }
    reduce_members<T>(c, lo, hi, sh, cnt, klo, khi);
  }
  if (cnt <= kMaxCand) return Refined{before, klo, khi, cnt, false};

  // one distinct key: a run of ties of equal mass, cut in cluster-index order
  int c = 0;
  u64 mm = 0;
#pragma unroll 1
  for (int e = 0; e < E; ++e) {
    const float le = logit(e);
    if (in_play<kCount>(mx - le) && ordered_key(le) == klo) {
      ++c;
      mm = mass_of<kCount>(mx - le);
    }
  }
  mm = wave_max(mm);
  if (lane_id() == 0) sh.scr64[wave_id()] = mm;
  __syncthreads();
  u64 m_tie = 0;
  {
    const int t = threadIdx.x & 15;
    m_tie = row16_max(t < (T / 64) ? sh.scr64[t] : 0ull);
  }
  __syncthreads();
  const u64 need = (tau - before + m_tie - 1) / m_tie;  // ties taken, 1 <= need <= cnt
  int tot;
  const int ex = block_excl_scan<int, (T / 64)>(c, sh.scri, tot);
  if ((u64)ex < need && need <= (u64)(ex + c)) {
    int seen = ex;
#pragma unroll 1
    for (int e = 0; e < E; ++e) {
      const float le = logit(e);
      if (in_play<kCount>(mx - le) && ordered_key(le) == klo) {
        ++seen;
        if ((u64)seen == need) {
          sh.res_key = klo;
          sh.res_idx = base + e;
          sh.res_mass = before + need * m_tie;
        }
      }
    }
  }
  __syncthreads();
  return Refined{before, klo, khi, cnt, true};
}

// Last element (key, index) of the shortest prefix of the order whose mass reaches tau
// (1 <= tau <= total mass) and that prefix's mass.  ex/hb: this thread's exclusive
// prefix and its consecutive bins of the level-1 histogram.  `slot` picks the candidate counter.
// cached_*: the bin whose members are currently gathered in sh.cand_* (reused when the
// second threshold falls into the same bin).  Block-uniform control flow.
template <int E, bool kCount, int T>
__device__ __forceinline__ void find_prefix(const float (&l)[E], const float *lg, int kc, float mx, float bs, int base, u64 masked, u64 tau, u64 ex,
                                            const u64 (&hb)[bins_of(T) / T], int slot, Shared<T> &sh, int &cached_bin, int &cached_cnt,
                                            u64 &cached_before, uint32_t &key_o, int &idx_o, u64 &mass_o) {
  const int tid = threadIdx.x;
  constexpr int kBins = bins_of(T);
  {
    u64 run = ex;
#pragma unroll
    for (int q = 0; q < kBins / T; ++q) {
      if (run < tau && tau <= run + hb[q]) {
        sh.bin = (kBins / T) * tid + q;
        sh.before = run;
      }
      run += hb[q];
    }
  }
  __syncthreads();
  const int bin1 = sh.bin;
  u64 before = sh.before;
  int cnt;
  bool done = false;
  const bool reused = bin1 == cached_bin;
  if (reused) {
    cnt = cached_cnt;
    before = cached_before;
  } else {
    // gather the members of the crossing bin (bins are monotone in the logit)
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const float d = mx - l[e];
      if (in_play<kCount>(d) && level1_bin(d, bs, kBins) == bin1) {
        const int s = atomicAdd(&sh.ncand[slot], 1);
        if (s < kMaxCand) {
          sh.cand_key[s] = ordered_key(l[e]);
          sh.cand_idx[s] = base + e;
          sh.cand_m[s] = mass_of<kCount>(d);
          sh.cand_ahead[s] = 0;
        }
      }
    }
    __syncthreads();
    cnt = sh.ncand[slot];
    cached_bin = bin1;
    cached_cnt = cnt;
    cached_before = before;
    if (cnt > kMaxCand) {
      cached_bin = -1;  // the candidate arrays will not hold this bin
      const Refined rf = refine_or_cut_ties<E, kCount, T>(lg, kc, mx, bs, base, bin1, tau, before, masked, &sh);
      const uint32_t klo = rf.klo, khi = rf.khi;
      before = rf.before;
      cnt = rf.cnt;
      done = rf.done;
      if (!done) {
        if (tid == 0) sh.ncand[slot] = 0;
        __syncthreads();
#pragma unroll
        for (int e = 0; e < E; ++e) {
          const uint32_t k = ordered_key(l[e]);
          if (in_play<kCount>(mx - l[e]) && k >= klo && k <= khi) {
            const int s = atomicAdd(&sh.ncand[slot], 1);
            sh.cand_key[s] = k;
            sh.cand_idx[s] = base + e;
            sh.cand_m[s] = mass_of<kCount>(mx - l[e]);
            sh.cand_ahead[s] = 0;
          }
        }
        __syncthreads();
      }
    }
  }
  if (!done) {
    // Rank the members exactly on (key descending, index ascending).  The block is cut into slices of P threads
    // (P = the power of two that holds the members): thread i of slice s adds up the weight of the members of the
    // s-th part of the list that precede member i, and the slices' integer sums meet in sh.cand_ahead (any order
    // gives the same bits).  A bin that is still gathered from the first threshold keeps its sums.
    const int P = cnt <= 64 ? 64 : cnt <= 128 ? 128 : cnt <= 256 ? 256 : kMaxCand;
    const int n_slices = T > P ? T / P : 1, slice = T > P ? tid / P : 0;
    if (!reused) {
      const int ja = slice * cnt / n_slices, jb = (slice + 1) * cnt / n_slices;
      for (int i = tid & (P - 1); i < cnt; i += T) {
        const uint32_t ki = sh.cand_key[i];
        const int ii = sh.cand_idx[i];
        u64 part = 0;
#pragma unroll 4
        for (int j = ja; j < jb; ++j) {  // j is uniform in a wave: broadcast reads, four members in flight
          const uint32_t kj = sh.cand_key[j];
          const int ij = sh.cand_idx[j];
          const u64 mj = sh.cand_m[j];
          part += (kj > ki || (kj == ki && ij < ii)) ? mj : 0;
        }
        if (part) atomicAdd(&sh.cand_ahead[i], part);
      }
      __syncthreads();
    }
    for (int i = tid; i < cnt; i += T) {
      const u64 ahead = before + sh.cand_ahead[i], mi = sh.cand_m[i];
      if (ahead < tau && tau <= ahead + mi) {  // true for exactly one member
        sh.res_key = sh.cand_key[i];
        sh.res_idx = sh.cand_idx[i];
        sh.res_mass = ahead + mi;
      }
    }
    __syncthreads();
  }
  key_o = sh.res_key;
  idx_o = sh.res_idx;
  mass_o = sh.res_mass;
}

// Where the selected ids and the stage-3 plan of one head go: the caller-visible id list,
// and either the LDS lists of the inline attention or the global plan arrays.
// A store that workgroups of the SAME launch will read (coherent: it is performed at the memory side, not left in
// this compute die's L2), or a plain one for a later launch.
__device__ __forceinline__ void st_i32(int32_t *p, int32_t v, bool coherent) {
  if (coherent)
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else
    *p = v;
}

struct Emit {
  int32_t *sel, *ent_src, *row_start, *chunk_entry;
  int *l_start, *l_src;
  bool plan, to_lds;
  bool coherent;  // the global plan is read by the stage-3 queue of this same launch
  int n_ex, n_tok;
  // (The store to the id list comes last: the offset of a cluster may still be on its way from memory when the
  // entry is written, and a wait for it that follows a store also waits for that store to complete.)
  __device__ __forceinline__ void exact(int pe, int pt, int sz, int off, int id) const {
    if (plan) {
      if (to_lds) {
        l_start[pe] = pt;
        l_src[pe] = off;
      } else {
        st_i32(ent_src + pe, off, coherent);
        st_i32(row_start + pe, pt, coherent);
        for (int q = (pt + kChunkRows - 1) / kChunkRows; q * kChunkRows < pt + sz; ++q) st_i32(chunk_entry + q, pe, coherent);
      }
    }
    sel[pe] = id;
  }
  __device__ __forceinline__ void approx(int pa, int id) const {
    const int j = n_ex + pa, row = n_tok + pa;
    if (plan) {
      if (to_lds) {
        l_start[j] = row;
        l_src[j] = id;
      } else {
        st_i32(ent_src + j, id, coherent);
        st_i32(row_start + j, row, coherent);
        if (row % kChunkRows == 0) st_i32(chunk_entry + row / kChunkRows, j, coherent);
      }
    }
    sel[j] = id;
  }
};

// The two thresholds of a head in units of the rule's weights.
//   first : all == true, or tau1 in [1, W]
//   second: kind 0 = nothing exact, 1 = every retained cluster, 2 = tau2 in [1, m1]
template <bool kCount>
__device__ __forceinline__ bool retain_all(const SelectArgs &a, u64 W) {
  return kCount ? (u64)a.k_retained >= W : a.p1 >= 1.0f;
}
template <bool kCount>
__device__ __forceinline__ u64 first_tau(const SelectArgs &a, u64 W) {
  if (kCount) return (u64)a.k_retained < W ? (u64)a.k_retained : W;  // k_retained >= 1 here
  return top_p_first_tau(a.p1, W);
}
// m1: weight of the retained prefix
template <bool kCount>
__device__ __forceinline__ int second_tau(const SelectArgs &a, u64 W, u64 m1, u64 &tau2) {
  if (kCount) {
    if (a.k_exact <= 0) return 0;
    if ((u64)a.k_exact >= m1) return 1;
    tau2 = (u64)a.k_exact;
    return 2;
  }
  return top_p_second_tau(a.p2, a.p2_absolute != 0, W, m1, tau2);
}

// One wave ranks a top set held one entry per lane (act: this lane holds one; key, index, mass, size, offset; an
// entry of mass 0 is a pinned cluster) pairwise on (key descending, index ascending) and, if the set holds the first
// threshold's weight, emits both lists in ascending cluster index and leaves the three counts in sh.f_*.
// Otherwise sh.f_nex = -1 and nothing is emitted.  W: total weight of the head.  Call from every lane of one wave;
// the caller's barrier publishes the result.
template <bool kCount, int T>
__device__ __forceinline__ void rank_lanes(const SelectArgs &a, Shared<T> &sh, Emit &emit, bool act, uint32_t key_i,
                                           int idx_i, u64 m_i, int sz_i, int off_i, u64 W, bool can_inline) {
  const u64 members = __ballot(act);
  if (!act) {
    key_i = 0u;
    idx_i = INT_MAX;
    m_i = 0;
    sz_i = 0;
  }
  const bool pin_i = act && m_i == 0;  // a candidate of the top set has weight > 0, a pinned cluster 0
  const u64 tau1 = first_tau<kCount>(a, W);
  // lane j holds entry j: the loops below fetch it with readlane (j is uniform), not from LDS.  A top set has a
  // handful of members, so the sums over it are taken in these loops on uniform values (scalar arithmetic) instead
  // of by 64-lane reductions, each of which is a chain of a few dozen dependent vector instructions.
  const uint32_t mlo_i = (uint32_t)m_i, mhi_i = (uint32_t)(m_i >> 32);
  auto mass_of_lane = [&](int j) {
    return ((u64)(uint32_t)__builtin_amdgcn_readlane(mhi_i, j) << 32) | (uint32_t)__builtin_amdgcn_readlane(mlo_i, j);
  };
  u64 ahead = 0;  // mass of the clusters that precede cluster i in the order
  u64 in_set = 0;  // weight of the whole top set
  for (u64 mm = members; mm; mm &= mm - 1) {
    const int j = __builtin_ctzll(mm);
    const uint32_t kj = __builtin_amdgcn_readlane(key_i, j);
    const int ij = __builtin_amdgcn_readlane(idx_i, j);
    const u64 mj = mass_of_lane(j);
    in_set += mj;
    if (kj > key_i || (kj == key_i && ij < idx_i)) ahead += mj;
  }
  if (in_set < tau1) {  // integer sums: exact.  The retained set is not inside the top set.
    if (lane_id() == 0) sh.f_nex = -1;
    return;
  }
  const bool ret = pin_i || (act && ahead < tau1);
  u64 m1 = 0;  // mass of the retained prefix
  for (u64 mm = __ballot(ret && !pin_i); mm; mm &= mm - 1) m1 += mass_of_lane(__builtin_ctzll(mm));
  u64 tau2 = 0;
  const int kind = second_tau<kCount>(a, W, m1, tau2);
  const bool exa = pin_i || (kind == 1 ? ret : (kind == 2 && act && ahead < tau2));
  const bool apx = ret && !exa;
  const u64 exa_mask = __ballot(exa), apx_mask = __ballot(apx);
  const int n_ex = __popcll(exa_mask), n_ap = __popcll(apx_mask);
  int n_tok = 0;
  // position of cluster i in its list = selected clusters with a smaller index
  int pe = 0, pa = 0, pt = 0;
  for (u64 mm = exa_mask | apx_mask; mm; mm &= mm - 1) {
    const int j = __builtin_ctzll(mm);
    const bool before = __builtin_amdgcn_readlane(idx_i, j) < idx_i;
    if ((exa_mask >> j) & 1) {
      const int sz_j = __builtin_amdgcn_readlane(sz_i, j);
      n_tok += sz_j;
      pe += before;
      pt += before ? sz_j : 0;
    } else {
      pa += before;
    }
  }
  emit.to_lds = can_inline && n_tok + n_ap <= inline_rows_of(T);
  emit.n_ex = n_ex;
  emit.n_tok = n_tok;
  if (exa) emit.exact(pe, pt, sz_i, off_i, idx_i);
  if (apx) emit.approx(pa, idx_i);
  if (lane_id() == 0) {
    sh.f_nex = n_ex;
    sh.f_nap = n_ap;
    sh.f_ntok = n_tok;
    if (emit.to_lds) emit.l_start[n_ex + n_ap] = n_tok + n_ap;  // the end of the row prefix: the lists are complete
  }
}

// the same for a top set gathered in sh.top_* (ntop <= kTopMax entries in any order)
template <bool kCount, int T>
__device__ __forceinline__ void rank_top_set(const SelectArgs &a, Shared<T> &sh, Emit &emit, int ntop, u64 W,
                                             bool can_inline) {
  const int i = lane_id();
  const bool act = i < ntop;
  rank_lanes<kCount, T>(a, sh, emit, act, act ? sh.top_key[i] : 0u, act ? sh.top_idx[i] : 0, act ? sh.top_m[i] : 0,
                        act ? sh.top_sz[i] : 0, act ? sh.top_off[i] : 0, W, can_inline);
}

// Marks a loaded value as used here.  The compiler waits for a load at the first use of its result; when that use
// sits in a branch behind stores, the wait (the counter of outstanding memory operations is shared and in order) also
// waits for those stores to complete, a full round trip on the critical path, and at the joins of skipped branches it
// has to assume the load is still outstanding.  A use right where the value has certainly arrived costs nothing.
__device__ __forceinline__ void arrived(int v) { asm volatile("" ::"v"(v)); }

// Top-p selection of a peaked head from the scoring kernel's sub-tile summaries, without reading the head's
// logits, by ONE wave and without a barrier: it reads (max, sum exp) of every sub-tile, which gives the max logit
// exactly and the total mass W (the sub-tile sums rescaled to the max and added up in fp32, per lane and then over
// the lanes, and brought into the 2^-40 fixed point of the other paths: W is within a few 1e-7 of the integer sum of
// the clusters' own masses, so a threshold p * W moves by that much).  Only sub-tiles whose max lies within kTopCut
// of the head's max can hold a member of the top set; if there are at most four of them, the wave reads their 64 logits, sizes and
// offsets (one cluster per lane) and ranks the top set in place.  Returns false (block-uniform) when the head is not
// peaked enough for that: then nothing has been emitted.
template <int T, bool kWarm>
__device__ __forceinline__ bool lite_select(const SelectArgs &a, Shared<T> &sh, Emit &emit, int c0, int kc,
                                            const float *lg, bool plan, bool can_inline, int64_t seg_row0,
                                            int (&warm)[4], int &n_ex, int &n_ap, int &n_tok) {
  const int tid = threadIdx.x;
  if (tid < 64) {
    const int n_sub = (kc + kSubTile - 1) / kSubTile;
    const float2 *sp = a.summaries + (int64_t)blockIdx.x * a.sub_stride;
    float2 sv[kLiteSubPerLane];
#pragma unroll
    for (int i = 0; i < kLiteSubPerLane; ++i) {
      const int u = tid + 64 * i;
      sv[i] = u < n_sub ? sp[u] : make_float2(-INFINITY, 0.f);
    }
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < kLiteSubPerLane; ++i) m = fmaxf(m, sv[i].x);
    const float M = wave_max(m);
    // The sub-tiles that may hold a cluster within kTopCut of the max: a bit per own sub-tile in every lane, then the
    // few lanes that hold one are walked on uniform values (no LDS, no barrier); slot k of the list (any order) goes
    // to lanes 16 k .. + 15.
    uint32_t top_bits = 0;
#pragma unroll
    for (int i = 0; i < kLiteSubPerLane; ++i)
      if (sv[i].x > -INFINITY && M - sv[i].x < kTopCut) top_bits |= 1u << i;
    static_assert(kLiteMaxTopSub == 4, "the list below is four uniform values");
    int n_ts = 0, s0 = -1, s1 = -1, s2 = -1, s3 = -1;
    for (u64 lanes = __ballot(top_bits != 0); lanes && n_ts <= kLiteMaxTopSub; lanes &= lanes - 1) {
      const int j = __builtin_ctzll(lanes);
      for (uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)top_bits, j); b; b &= b - 1) {
        s3 = s2;
        s2 = s1;
        s1 = s0;
        s0 = j + 64 * __builtin_ctz(b);
        ++n_ts;
      }
    }
    bool ok = M > -INFINITY && n_ts <= kLiteMaxTopSub;  // no candidate at all, or a flat head: the general path
    if (ok) {
      const int slot = tid >> 4;
      const int my_sub = slot == 0 ? s0 : slot == 1 ? s1 : slot == 2 ? s2 : s3;  // -1: no such sub-tile
      const int i = my_sub * kSubTile + (tid & 15);
      const bool have = my_sub >= 0 && i < kc;
      // the second round of loads: all three issued together (nothing uses a value inside the branch, so no wait
      // separates them), and before the total mass is summed
      float l = -INFINITY;
      int sz = 0, off = 0;
      if (have) {
        l = lg[i];
        sz = a.cluster_sizes[c0 + i];
        off = plan ? a.cluster_offsets[c0 + i] : 0;
      }
      float acc = 0.f;
#pragma unroll
      for (int u = 0; u < kLiteSubPerLane; ++u)
        if (sv[u].x > -INFINITY) acc = fmaf(sv[u].y, __builtin_amdgcn_exp2f((sv[u].x - M) * kLog2e), acc);
      // fp32 over the lanes (a tree of depth 6), then the 2^-40 fixed point of the other paths
      const u64 W = (u64)((double)wave_sum(acc) * 1099511627776.0);
      l += 0.0f;  // -0 becomes +0
      arrived(sz);
      arrived(off);
      if (kWarm && can_inline) {
        // The cluster with the largest logit is exact whatever the thresholds are: its rows start their way from HBM
        // now, one touch per 64 bytes, and have arrived in the L2 when the lists are written and the rows are
        // attended (the values are never used; the caller marks them as arrived once the rows have been read).
        const u64 top = __ballot(have && l == M);
        const int j = top ? __builtin_ctzll(top) : 0;
        const int n4 = 4 * min(__builtin_amdgcn_readlane(top ? sz : 0, j), 32);
        const int64_t byte0 = (seg_row0 + __builtin_amdgcn_readlane(off, j)) * kRowBytes;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int piece = min(tid + 64 * u, n4 - 1);
          if (n4 > 0) {
            warm[2 * u] = *reinterpret_cast<const int *>(static_cast<const char *>(a.k_cache) + byte0 + 64 * piece);
            warm[2 * u + 1] = *reinterpret_cast<const int *>(static_cast<const char *>(a.v_cache) + byte0 + 64 * piece);
          }
        }
      }
      const float d = M - l;
      const bool member = have && d < kTopCut;
      rank_lanes<false, T>(a, sh, emit, member, ordered_key(l), i, member ? fx_mass(d) : 0, sz, off, W, can_inline);
    } else if (tid == 0) {
      sh.f_nex = -1;
    }
    if (tid == 0) sh.lite_max = M;
  }
  lds_barrier();
  if (sh.f_nex < 0) return false;
  n_ex = sh.f_nex;
  n_ap = sh.f_nap;
  n_tok = sh.f_ntok;
  return true;
}

__device__ __forceinline__ void put_counts(const SelectOut &o, int head, int n_exact, int n_retained, int n_tokens,
                                           bool coherent) {
  st_i32(o.n_exact + head, n_exact, coherent);
  st_i32(o.n_retained + head, n_retained, coherent);
  o.n_exact_tokens[head] = n_tokens;
  if (o.n_exact_copy) o.n_exact_copy[head] = n_exact;
  if (o.n_retained_copy) o.n_retained_copy[head] = n_retained;
  if (o.n_exact_tokens_copy) o.n_exact_tokens_copy[head] = n_tokens;
}

// A thread's E consecutive logits of the head and, with few logits per thread (kPre), the sizes and offsets of the
// same clusters next to them, so that no dependent load sits between the selection and the first K/V row.
template <int E>
struct HeadInputs {
  static constexpr bool kPre = E <= 8;
  static constexpr int EP = kPre ? E : 1;
  float l[E];
  int psz[EP], poff[EP];
};
template <int E>
__device__ __forceinline__ void load_head_inputs(const SelectArgs &a, int c0, int kc, const float *lg, bool plan,
                                                 HeadInputs<E> &in) {
  constexpr bool kPre = HeadInputs<E>::kPre;
  constexpr int EP = HeadInputs<E>::EP;
  const int base = threadIdx.x * E;
  float(&l)[E] = in.l;
  int(&psz)[EP] = in.psz;
  int(&poff)[EP] = in.poff;
  if (E >= 4 && (reinterpret_cast<uintptr_t>(lg) & 15) == 0 && base + E <= kc) {
    // the thread's whole run lies inside the segment: all its 16-byte loads go out back to back
#pragma unroll
    for (int e = 0; e < E; e += 4) {
      const float4 v = *reinterpret_cast<const float4 *>(lg + base + e);
      l[e] = v.x;
      l[e + 1 < E ? e + 1 : e] = v.y;
      l[e + 2 < E ? e + 2 : e] = v.z;
      l[e + 3 < E ? e + 3 : e] = v.w;
    }
  } else {
    // the ragged or unaligned case: unconditional loads at clamped indices, the values chosen afterwards (loads
    // inside a condition are waited for one by one: E dependent round trips)
#pragma unroll
    for (int e = 0; e < E; ++e) l[e] = -INFINITY;
    if (kc > 0) {
      float got[E];
#pragma unroll
      for (int e = 0; e < E; ++e) got[e] = lg[min(base + e, kc - 1)];
#pragma unroll
      for (int e = 0; e < E; ++e) l[e] = (base + e < kc) ? got[e] : -INFINITY;
    }
  }
  if (kPre) {
    const int32_t *sp = a.cluster_sizes + c0 + base, *op = a.cluster_offsets + c0 + base;
    if (E >= 4 && ((reinterpret_cast<uintptr_t>(sp) | reinterpret_cast<uintptr_t>(op)) & 15) == 0 && base + E <= kc) {
#pragma unroll
      for (int e = 0; e < EP; e += 4) {
        const int4 v = *reinterpret_cast<const int4 *>(sp + e);
        psz[e] = v.x; psz[e + 1 < EP ? e + 1 : e] = v.y; psz[e + 2 < EP ? e + 2 : e] = v.z; psz[e + 3 < EP ? e + 3 : e] = v.w;
        if (plan) {
          const int4 u = *reinterpret_cast<const int4 *>(op + e);
          poff[e] = u.x; poff[e + 1 < EP ? e + 1 : e] = u.y; poff[e + 2 < EP ? e + 2 : e] = u.z; poff[e + 3 < EP ? e + 3 : e] = u.w;
        }
      }
    } else {
#pragma unroll
      for (int e = 0; e < EP; ++e) psz[e] = poff[e] = 0;
      if (kc > 0) {
        const int32_t *s0 = a.cluster_sizes + c0, *o0 = a.cluster_offsets + c0;
        int gs[EP], go[EP];
#pragma unroll
        for (int e = 0; e < EP; ++e) {
          gs[e] = s0[min(base + e, kc - 1)];
          go[e] = plan ? o0[min(base + e, kc - 1)] : 0;
        }
#pragma unroll
        for (int e = 0; e < EP; ++e) {
          psz[e] = (base + e < kc) ? gs[e] : 0;
          poff[e] = (base + e < kc) ? go[e] : 0;
        }
      }
    }
  }
}

// The selection proper for one head (one workgroup) on the thread's loaded inputs: fast path for a peaked head,
// general threshold search otherwise; emits the lists (and the plan) and returns the three counts.  Returns false
// when the head had no candidate at all and has been finished here (counts, zero output).  known_max: the head's max
// logit if the caller has it already (NaN if not).  inline_limit: the most rows of this head that are worth
// attending in this workgroup (a head that took the general path has used up its time: 64 rows, which four waves
// attend in one round of loads; a longer list goes to the split decode).
template <int E, bool kCount, int T>
__device__ __forceinline__ bool full_select(const SelectArgs &a, Shared<T> &sh, Emit &emit, int head, int c0, int kc,
                                            const float *lg, bool plan, bool can_inline, HeadInputs<E> &in,
                                            float known_max, int &n_ex, int &n_ap, int &n_tok, int &inline_limit) {
  constexpr int kBins = bins_of(T);
  constexpr bool kPre = HeadInputs<E>::kPre;
  constexpr int kGeneralInlineRows = 64;
  const int tid = threadIdx.x;
  const int base = tid * E;
  float(&l)[E] = in.l;
  int(&psz)[HeadInputs<E>::EP] = in.psz;
  int(&poff)[HeadInputs<E>::EP] = in.poff;
  inline_limit = inline_rows_of(T);
  // Pinned clusters (the caller's sink / window tokens): their logits leave the distribution here and
  // they join the exact list further down.  bit e of pinmask: element e is a pinned, non-empty cluster.
  u64 pinmask = 0, flagged = 0;  // flagged: every element that carries the flag, empty clusters included
  const bool has_flags = a.cluster_flags != nullptr;
  if (has_flags) {
    const uint8_t *fp = a.cluster_flags + c0 + base;
    constexpr int kVec = E < 8 ? E : 8;  // flag bytes per load when the thread's run of flags is aligned
    if ((reinterpret_cast<uintptr_t>(fp) & (kVec - 1)) == 0 && base + E <= kc) {
#pragma unroll
      for (int e = 0; e < E; e += kVec) {
        u64 w;
        if (kVec == 8) w = *reinterpret_cast<const u64 *>(fp + e);
        else if (kVec == 4) w = *reinterpret_cast<const uint32_t *>(fp + e);
        else w = *reinterpret_cast<const uint16_t *>(fp + e);
#pragma unroll
        for (int u = 0; u < kVec; ++u) pinmask |= ((w >> (8 * u)) & 1ull) << (e + u);
      }
    } else {
#pragma unroll
      for (int e = 0; e < E; ++e)
        if (base + e < kc && (fp[e] & 1u)) pinmask |= 1ull << e;
    }
    flagged = pinmask;
#pragma unroll
    for (int e = 0; e < E; ++e)
      if ((pinmask >> e) & 1) {
        const int sz = kPre ? psz[kPre ? e : 0] : a.cluster_sizes[c0 + base + e];
        if (sz <= 0) pinmask &= ~(1ull << e);
        l[e] = -INFINITY;
      }
  }
  // With the max known, the level-1 histogram has been cleared (and published) by the caller and is filled while the
  // weights are summed (one evaluation of the masses instead of two).
  const bool hist_early = !kCount && known_max == known_max;
  if (!hist_early)
    for (int i = tid; i < kBins; i += T) sh.hist[i] = 0;
  if (tid < 2) sh.ncand[tid] = 0;
  if (tid == 2) sh.ntop = 0;
  float tmax = -INFINITY;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    l[e] += 0.0f;  // -0 becomes +0
    tmax = fmaxf(tmax, l[e]);
  }
  // (the barriers of the block max, or else the one of the weight sums below, also publish the zeroed LDS)
  const float mx_raw = known_max == known_max ? known_max + 0.0f : block_max<(T / 64)>(tmax, sh.scrf);
  // no candidate cluster, or a budget of 0: the distribution selects nothing
  const bool nothing = mx_raw == -INFINITY || (kCount && a.k_retained <= 0);
  const float mx = mx_raw == -INFINITY ? 0.f : mx_raw;
  if (nothing && !has_flags) {  // and nothing can be pinned: zero output
    if (tid == 0) {
      put_counts(a.out, head, 0, 0, 0, emit.coherent);
      if (plan) {
        st_i32(emit.row_start, 0, emit.coherent);
        st_i32(a.plan.head_rows + head, 0, emit.coherent);
        st_i32(a.plan.done + head, 0, emit.coherent);
      }
      if (can_inline && a.lse) a.lse[head] = -INFINITY;
    }
    if (can_inline && tid < kHeadDim) store_out(a.attn_out, a.out_is_bf16, head, tid, 0.f);
    return false;
  }

  // level-1 bins: top-p spreads them over the kCut below the max that carries mass; a fixed budget
  // spreads them over the head's whole range of finite logits
  float bs = (float)kBins / kCut;
  if (kCount) {
    float tmin = INFINITY;
#pragma unroll
    for (int e = 0; e < E; ++e) tmin = fminf(tmin, l[e] == -INFINITY ? INFINITY : l[e]);
    const float mn = -block_max<(T / 64)>(-tmin, sh.scrf);
    bs = mx > mn ? ((float)kBins - 0.5f) / (mx - mn) : 0.f;
  }

  // ---- total mass; how many clusters are close to the top ------------------
  u64 wsum = 0, wtop = 0;
  int ctop = 0;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const float d = mx - l[e];
    if (in_play<kCount>(d)) {
      const u64 m = mass_of<kCount>(d);
      wsum += m;
      if (d < kTopCut) {
        ++ctop;
        wtop += m;
      }
      if (hist_early && m) atomicAdd(&sh.hist[level1_bin(d, bs, kBins)], m);
    }
  }
  ctop += __popcll(pinmask);  // pinned clusters ride along in the top set
  int ntop;
  u64 W, Wtop;  // total weight (top-p: >= 2^40, the max element has weight 1; fixed budget: the non-empty clusters), weight of the top set
  {
    wsum = wave_sum(wsum);
    wtop = wave_sum(wtop);
    ctop = wave_sum(ctop);
    if (lane_id() == 0) {
      sh.scr64[wave_id()] = wsum;
      sh.scr64b[wave_id()] = wtop;
      sh.scri[wave_id()] = ctop;
    }
    __syncthreads();
    W = partials_sum<u64, (T / 64)>(sh.scr64);
    Wtop = partials_sum<u64, (T / 64)>(sh.scr64b);
    ntop = partials_sum<int, (T / 64)>(sh.scri);
  }
  if (kPre) {  // loaded next to the logits, long here: no wait for them between the stores of the emission
#pragma unroll
    for (int e = 0; e < HeadInputs<E>::EP; ++e) {
      arrived(psz[e]);
      arrived(poff[e]);
    }
  }

  const bool all = !nothing && retain_all<kCount>(a, W);  // every non-empty candidate is retained
  // fast path: the top set is small and already holds the first threshold's weight (integer sums: exact), so
  // the retained set lies inside it (the usual case for a peaked head)
  const bool fast = !nothing && !all && ntop <= kTopMax && Wtop >= first_tau<kCount>(a, W);
  if (fast) {
    // ---- gather the top set with its sizes / offsets, then one wave ranks it pairwise ----
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const float d = mx - l[e];
      if (d < kTopCut || ((pinmask >> e) & 1)) {
        const int s = atomicAdd(&sh.ntop, 1);
        const int i = base + e;
        sh.top_key[s] = ordered_key(l[e]);
        sh.top_idx[s] = i;
        sh.top_m[s] = mass_of<kCount>(d);
        sh.top_sz[s] = kPre ? psz[kPre ? e : 0] : a.cluster_sizes[c0 + i];
        sh.top_off[s] = !plan ? 0 : kPre ? poff[kPre ? e : 0] : a.cluster_offsets[c0 + i];
      }
    }
    __syncthreads();
    if (wave_id() == 0) rank_top_set<kCount, T>(a, sh, emit, ntop, W, can_inline);  // holds the weight: always emits
    __syncthreads();
    n_ex = sh.f_nex;
    n_ap = sh.f_nap;
    n_tok = sh.f_ntok;
  }

  if (!fast) {
    // the prefix ends: the last retained and the last exact cluster of the order as (key, index); the
    // initial values select nothing
    uint32_t key1 = 0xffffffffu, key2 = 0xffffffffu;
    int idx1 = -1, idx2 = -1;
    if (!nothing) {
      // ---- general path: level-1 mass histogram, scan, threshold search ---------
      if (!hist_early) {
#pragma unroll
        for (int e = 0; e < E; ++e) {
          const float d = mx - l[e];
          const u64 m = mass_of<kCount>(d);
          if (m) atomicAdd(&sh.hist[level1_bin(d, bs, kBins)], m);
        }
        __syncthreads();
      }
      constexpr int B = kBins / T;  // consecutive bins per thread
      u64 hb[B], hsum = 0;
#pragma unroll
      for (int q = 0; q < B; ++q) {
        hb[q] = sh.hist[B * tid + q];
        hsum += hb[q];
      }
      u64 Wh;  // equals W: the same masses, summed in another order
      const u64 ex = block_excl_scan<u64, (T / 64)>(hsum, sh.scr64, Wh);

      u64 mass1;
      int cached_bin = -1, cached_cnt = 0;
      u64 cached_before = 0;
      if (all) {  // every non-empty cluster
        key1 = kKeyLowestFinite;
        idx1 = INT_MAX;
        mass1 = W;
      } else {
        find_prefix<E, kCount, T>(l, lg, kc, mx, bs, base, flagged, first_tau<kCount>(a, W), ex, hb, 0, sh, cached_bin, cached_cnt,
                               cached_before, key1, idx1, mass1);
      }
      u64 tau2 = 0;
      const int kind = second_tau<kCount>(a, W, mass1, tau2);
      if (kind == 1) {
        key2 = key1;
        idx2 = idx1;
      } else if (kind == 0) {  // nothing is exact
        key2 = 0xffffffffu;
        idx2 = -1;
      } else {
        u64 mass2;
        __syncthreads();  // sh.bin / sh.res_* of the first search have been read by every thread
        find_prefix<E, kCount, T>(l, lg, kc, mx, bs, base, flagged, tau2, ex, hb, 1, sh, cached_bin, cached_cnt, cached_before, key2, idx2,
                               mass2);
      }

    }
    // ---- compaction in ascending cluster index ------------------------------
    // Only clusters in play (non-zero weight) can be selected, unless all non-empty ones are.
    u64 exa_mask = 0, ret_mask = 0;  // bit e: element e of this thread is exact / approximated
    int te = 0;                      // tokens of this thread's exact clusters
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const uint32_t k = ordered_key(l[e]);
      const int i = base + e;
      const bool live = all ? l[e] != -INFINITY : in_play<kCount>(mx - l[e]);
      const bool exa = ((pinmask >> e) & 1) || (live && (k > key2 || (k == key2 && i <= idx2)));
      const bool apx = live && !exa && (k > key1 || (k == key1 && i <= idx1));
      exa_mask |= (u64)exa << e;
      ret_mask |= (u64)apx << e;
      // sizes: preloaded, or fetched here for the sum and again (cached) when the entry is written
      if (exa) te += kPre ? psz[kPre ? e : 0] : a.cluster_sizes[c0 + i];
    }
    const int ce = __popcll(exa_mask), ca = __popcll(ret_mask);
    int pe, pa, pt;
    {
      // one barrier for the three counters: wave scans, wave totals through LDS, combined by 16-lane rows
      const int w = wave_id();
      const int ie = wave_incl_scan(ce), ia = wave_incl_scan(ca), it = wave_incl_scan(te);
      if (lane_id() == 63) {
        sh.scri[w] = ie;
        sh.scri[(T / 64) + w] = ia;
        sh.scri[2 * (T / 64) + w] = it;
      }
      __syncthreads();
      const int t16 = tid & 15;
      const bool has = t16 < (T / 64), mine = t16 < w;
      const int se = has ? sh.scri[t16] : 0, sa = has ? sh.scri[(T / 64) + t16] : 0, st = has ? sh.scri[2 * (T / 64) + t16] : 0;
      n_ex = row16_sum(se);
      n_ap = row16_sum(sa);
      n_tok = row16_sum(st);
      pe = row16_sum(mine ? se : 0) + ie - ce;
      pa = row16_sum(mine ? sa : 0) + ia - ca;
      pt = row16_sum(mine ? st : 0) + it - te;
    }
    inline_limit = kGeneralInlineRows;
    emit.to_lds = can_inline && n_tok + n_ap <= kGeneralInlineRows;
    emit.n_ex = n_ex;
    emit.n_tok = n_tok;
    if (ce + ca > 0) {
#pragma unroll
      for (int e = 0; e < E; ++e) {
        if ((exa_mask >> e) & 1) {
          const int sz = kPre ? psz[kPre ? e : 0] : a.cluster_sizes[c0 + base + e];
          const int off = !plan ? 0 : kPre ? poff[kPre ? e : 0] : a.cluster_offsets[c0 + base + e];
          emit.exact(pe, pt, sz, off, base + e);
          ++pe;
          pt += sz;
        } else if ((ret_mask >> e) & 1) {
          emit.approx(pa, base + e);
          ++pa;
        }
      }
    }
  }

  return true;
}

// Arrival of a head at the launch's `planned` counter (kGate): everything the stage-3 queue of this launch reads
// of the head has been stored coherently and has completed (the caller sees to that) before the counter moves.
// One word counts both: the low 16 bits the heads that have arrived, the high 16 bits those among them that
// left rows to the queue.  Returns the word as it was before this head: the caller must not touch that value
// before the head is done (a use is a wait for the counter's round trip).
constexpr int kQueueBit = 0x10000;
__device__ __forceinline__ int head_planned(int32_t *planned, bool needs_queue) {
  return __hip_atomic_fetch_add(planned, 1 + (needs_queue ? kQueueBit : 0), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Stage 2 for one head by one workgroup, and stage 3 too when the head has few rows.  kGate: the stage-3 queue for
// the heavier heads runs inside this same launch (select_decode_kernel): the plan, the counts and head_rows are then
// stored coherently, and the head reports to `planned` once they have completed; the first thread of the LAST wave
// (thread T - 64, which has nothing to load when the head has few rows, so the counter's round trip delays nobody)
// gets the counter word as it was before this head, with bit 31 set if the head left rows to the queue (-1 in the
// other threads).
template <int E, bool kCount, int T, bool kGate>
__device__ __forceinline__ int select_head(const SelectArgs &a, Shared<T> &sh, int32_t *planned) {
  constexpr int kInlineRows = inline_rows_of(T);
  const int head = blockIdx.x;
  const int b = head / a.n_q_heads, h = head % a.n_q_heads;
  const int seg = b * a.n_kv_heads + h / a.group;
  int c0, kc;
  if (a.uniform_kc > 0) {
    c0 = seg * a.uniform_kc;
    kc = a.uniform_kc;
  } else {
    c0 = a.seg_cluster_ptr[seg];
    kc = a.seg_cluster_ptr[seg + 1] - c0;
  }
  const float *lg = a.logits + (int64_t)a.group * c0 + (int64_t)(h % a.group) * kc;
  const int tid = threadIdx.x;
  int arrival = -1;

  const bool plan = a.plan.ent_src != nullptr;
  const bool can_inline = plan && a.attn_out != nullptr;
  Emit emit;
  emit.sel = a.out.sel_ids + (int64_t)head * a.max_k;
  emit.ent_src = plan ? a.plan.ent_src + (int64_t)head * a.max_k : nullptr;
  emit.row_start = plan ? a.plan.row_start + (int64_t)head * (a.max_k + 1) : nullptr;
  emit.chunk_entry = plan ? a.plan.chunk_entry + (int64_t)head * a.plan.chunk_stride : nullptr;
  emit.l_start = sh.at.l_start;
  emit.l_src = sh.at.l_src;
  emit.plan = plan;
  emit.coherent = kGate;

  // the item counter of the head's slab: cleared here for a decode launch that follows; with the queue in this
  // same launch the scoring kernel has cleared it (a plain store here could be written back over claims)
  if (!kGate && plan && tid == 0 && head % kMaxQueueHeads == 0) a.plan.queue_next[head / kMaxQueueHeads] = 0;
  const int64_t seg_row0 = can_inline ? a.seg_row_base[seg] : 0;  // needed last; its latency hides behind the selection

  int n_ex = 0, n_ap = 0, n_tok = 0, inline_limit = kInlineRows;
  // A peaked head is selected from the scoring kernel's summaries by the first wave; any other head by the search
  // over all its logits.  (Fetching the logits in the other waves while the first one tries was measured: their
  // loads queue in front of the first wave's own on the same CU and cost a peaked head 1.8 us.)
  const bool try_lite = !kCount && a.summaries && !a.cluster_flags && a.p1 < 1.0f && kc > 0 &&
                        kc <= kLiteSubPerLane * 64 * kSubTile;
  bool chosen = false;
  int warm[4] = {0, 0, 0, 0};  // rows fetched ahead by the summary path (never used)
  float known_max = __builtin_nanf("");
  if (try_lite) {
    // (the kernels for more than 8192 clusters per segment have no registers to spare for the rows fetched ahead)
    chosen = lite_select<T, (E <= 8)>(a, sh, emit, c0, kc, lg, plan, can_inline, seg_row0, warm, n_ex, n_ap, n_tok);
    if (!chosen) {  // the general path knows the max: it fills its histogram while it sums the weights
      known_max = sh.lite_max;
      for (int i = tid; i < bins_of(T); i += T) sh.hist[i] = 0;
      __syncthreads();
    }
  }
  HeadInputs<E> in;
  if (!chosen) load_head_inputs<E>(a, c0, kc, lg, plan, in);
  if (!chosen && !full_select<E, kCount, T>(a, sh, emit, head, c0, kc, lg, plan, can_inline, in, known_max, n_ex, n_ap,
                                            n_tok, inline_limit)) {
    // no candidate: finished inside (zero output, zero counts)
    if (kGate) {
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();  // thread 0's stores have completed
      if (tid == T - 64) arrival = head_planned(planned, false);
    }
    return arrival;
  }

  const int R = n_tok + n_ap;
  const bool inline_attn = can_inline && R <= inline_limit;
  if (tid == 0) {
    // a head that is attended here leaves nothing for the queue to read: its stores stay plain
    put_counts(a.out, head, n_ex, n_ex + n_ap, n_tok, kGate && !inline_attn);
    if (plan) {
      if (inline_attn) {
        if (!chosen) sh.at.l_start[n_ex + n_ap] = R;  // (the one-wave paths have written it with the lists)
        // attended here: nothing left for the stage-3 queue (kGate: head_rows was cleared by the scoring kernel)
        if (!kGate) a.plan.head_rows[head] = -1;
      } else {
        st_i32(emit.row_start + n_ex + n_ap, R, kGate);
        st_i32(a.plan.head_rows + head, R, kGate);
        if (!kGate && a.plan.pending && R > 0) atomicAdd(&a.plan.pending[head / kMaxQueueHeads], 1);
      }
      if (!kGate || !inline_attn) st_i32(a.plan.done + head, 0, kGate);
    }
  }
  // a head that is attended here has nothing to publish: it reports at once, and the workgroups that wait for the
  // count leave while it attends
  if (kGate && inline_attn && tid == T - 64) arrival = head_planned(planned, false);
  if (!inline_attn) {
    if (kGate) {  // the plan was written by every thread: all of it has completed before the head reports
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
      if (tid == T - 64) arrival = head_planned(planned, R > 0) | (R > 0 ? (int)0x80000000 : 0);
    }
    return arrival;
  }
  if (R == 0) {  // nothing to attend to: zero output
    if (tid < kHeadDim) store_out(a.attn_out, a.out_is_bf16, head, tid, 0.f);
    if (tid == 0 && a.lse) a.lse[head] = -INFINITY;
    return arrival;
  }

  // ---- inline attention for a head with few rows ---------------------------
  // the lists are in LDS (a head selected from the summaries: since the barrier that ended that selection); the
  // head's report to the counter (kGate) may still be in flight
  if (!chosen) lds_barrier();
  {
    const int lane16 = tid & 15, grp = tid >> 4;
    const uint4 qv = load_row_slice(a.q, (int64_t)head, lane16);
    RowSources src;
    src.k_cache = a.k_cache;
    src.v_cache = a.v_cache;
    src.k_centroids = a.k_centroids;
    src.v_centroids = a.v_centroids;
    src.seg_sizes = a.cluster_sizes + c0;
    src.seg_row0 = seg_row0;
    src.c0 = c0;
    RowState st;
    row_state_init(st);
    constexpr int kGroups = T / 16;
    const int per = kAttendBatch * ((R + kGroups * kAttendBatch - 1) / (kGroups * kAttendBatch));
    const int ra = grp * per, rb = min(R, ra + per);
    attend_rows(st, qv, a.scale_log2, src, sh.at.l_start, sh.at.l_src, n_ex + n_ap, 0, n_ex, ra, rb, kAttendBatch, lane16);
#pragma unroll
    for (int u = 0; u < 4; ++u) arrived(warm[u]);  // loads complete in order: these have, with the rows read above
    float M, L, o;
    const int groups_used = (R + per - 1) / per;
    block_merge<(T / 64)>(st, sh.at.m_m, sh.at.m_l, sh.at.m_acc, (groups_used + 3) / 4, M, L, o);
    if (tid < kHeadDim) {
      store_out(a.attn_out, a.out_is_bf16, head, tid, o / L);
      if (a.lse && tid == 0) a.lse[head] = (M + log2f(L)) * kLn2;
    }
  }
  return arrival;
}

template <int E, bool kCount, int T>
__global__ __launch_bounds__(T) void select_kernel(SelectArgs a) {
  __shared__ Shared<T> sh;
  select_head<E, kCount, T, false>(a, sh, nullptr);
}

// Stage 2 and stage 3 in one launch, for launches that serve few heads (a separate decode launch that finds nothing
// to do would cost as much as the selection itself).  Workgroup b < n_heads selects head b (and attends it if it has
// few rows); every workgroup, the ones beyond n_heads included, then serves the stage-3 queue of the heads that
// were left over.  The queue may only start when every head has reported to `planned`.  Nobody waits without
// bound: a selecting workgroup whose head was attended inline leaves when it is done; the one whose arrival completes
// the count serves the queue until it is empty (so all items are attended whoever else has left); the workgroups
// beyond n_heads and the ones whose own head left rows poll the counter for a limited time, serve the queue if the
// count is reached and leave if it is not.  The scoring kernel of
// the step clears planned and the item counter.
constexpr int kGatePolls = 20000;  // a microsecond or two each
struct QueueArgs {  // what the stage-3 queue needs beyond the selection's own arguments
  float *partials;
  int32_t *planned;
  int32_t splits, n_heads;
};
template <int E, bool kCount, int T>
__global__ __launch_bounds__(T) void select_decode_kernel(SelectArgs a, QueueArgs qa) {
  __shared__ Shared<T> sh;
  DP_DECODE_LDS(T);
  __shared__ int s_go;
  int32_t *const planned = qa.planned;
  const int n_heads = qa.n_heads;
  if ((int)blockIdx.x < n_heads) {
    const int word = select_head<E, kCount, T, true>(a, sh, planned);
    if (threadIdx.x == T - 64) {
      // the last head in serves the queue if any head (itself included) left rows to it
      bool go = (word & 0xffff) == n_heads - 1 && (word & 0xffff0000) != 0;
      if (!go && word != -1 && (word & (int)0x80000000)) {
        // a head that left rows: its workgroup stays for the queue like the ones beyond n_heads (a step of flat
        // heads would otherwise be served by those alone)
        int seen = 0;
#pragma unroll 1
        for (int it = 0; it < kGatePolls; ++it) {
          seen = __hip_atomic_load(planned, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if ((seen & 0xffff) >= n_heads) break;
          __builtin_amdgcn_s_sleep(64);
        }
        go = (seen & 0xffff) >= n_heads;
      }
      s_go = go;
    }
  } else if (threadIdx.x == 0) {
    int word = 0;
#pragma unroll 1
    for (int it = 0; it < kGatePolls; ++it) {
      word = __hip_atomic_load(planned, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if ((word & 0xffff) >= n_heads) break;
      __builtin_amdgcn_s_sleep(64);
    }
    s_go = (word & 0xffff) >= n_heads && (word >> 16) > 0;
  }
  __syncthreads();
  if (!s_go) return;
  // the queue's view of the same arguments
  DecodeArgs d;
  d.q = a.q;
  d.k_cache = a.k_cache;
  d.v_cache = a.v_cache;
  d.k_centroids = a.k_centroids;
  d.v_centroids = a.v_centroids;
  d.seg_row_base = a.seg_row_base;
  d.seg_cluster_ptr = a.seg_cluster_ptr;
  d.cluster_sizes = a.cluster_sizes;
  d.n_exact = a.out.n_exact;
  d.n_retained = a.out.n_retained;
  d.plan = a.plan;
  d.partials = qa.partials;
  d.out = a.attn_out;
  d.lse = a.lse;
  d.n_kv_heads = a.n_kv_heads;
  d.n_q_heads = a.n_q_heads;
  d.group = a.group;
  d.max_k = a.max_k;
  d.splits = qa.splits;
  d.out_is_bf16 = a.out_is_bf16;
  d.head0 = 0;
  d.n_heads = n_heads;
  d.queue_next = a.plan.queue_next;
  d.pending = nullptr;
  d.k_gather = d.v_gather = nullptr;
  d.rows_cap = 0;
  d.scale_log2 = a.scale_log2;
  decode_queue<T, false, true>(d, DP_DECODE_LDS_ARGS);
}

// ---- plan from caller-given sets (staged API) -----------------------------
constexpr int kPlanThreads = 256;

struct PlanArgs {
  const int32_t *seg_cluster_ptr, *cluster_sizes, *cluster_offsets;
  const int32_t *sel_ids, *n_exact, *n_retained;
  int32_t *n_exact_tokens;  // nullable
  int32_t n_kv_heads, n_q_heads, group, max_k;
  Plan plan;
  void *attn_out;  // a head without rows gets out = 0, lse = -inf here
  float *lse;
  int32_t out_is_bf16;
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
  if (tid == 0 && head % kMaxQueueHeads == 0) a.plan.queue_next[head / kMaxQueueHeads] = 0;

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
  const int R = n_tok + (n_rt - n_ex);
  if (tid == 0) {
    row_start[n_rt] = R;
    a.plan.head_rows[head] = R;
    a.plan.done[head] = 0;
    if (a.n_exact_tokens) a.n_exact_tokens[head] = n_tok;
    if (R == 0 && a.lse) a.lse[head] = -INFINITY;
  }
  if (R == 0 && a.attn_out && tid < kHeadDim) store_out(a.attn_out, a.out_is_bf16, head, tid, 0.f);
}

// with a queue: more workgroups than heads
template <int E, int T>
void launch_select_e(const SelectArgs &a, bool by_count, dim3 grid, hipStream_t s, hipEvent_t start, hipEvent_t stop,
                     const QueueArgs *queue) {
  if (queue) {
    // as many workgroups as 256 CUs hold at once (what the kernel's registers and LDS allow, asked once per
    // kernel): a workgroup that had to wait for a place would only find the count complete and leave, at the
    // launch's expense (with twice the resident number, a step of peaked heads over 2048 clusters took 11.8 us
    // in the mean and 14.5 us in every tenth step)
    static int per_cu[2] = {0, 0};
    int &n = per_cu[by_count ? 1 : 0];
    if (n == 0) {
      int got = 0;
      const hipError_t e =
          by_count ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&got, select_decode_kernel<E, true, T>, T, 0)
                   : hipOccupancyMaxActiveBlocksPerMultiprocessor(&got, select_decode_kernel<E, false, T>, T, 0);
      n = (e == hipSuccess && got > 0) ? got : 1;
    }
    const unsigned resident = 256u * (unsigned)n;
    const dim3 g(grid.x + 32 > resident ? grid.x + 32 : resident);
    if (start || stop) {
      if (by_count)
        hipExtLaunchKernelGGL((select_decode_kernel<E, true, T>), g, dim3(T), 0, s, start, stop, 0, a, *queue);
      else
        hipExtLaunchKernelGGL((select_decode_kernel<E, false, T>), g, dim3(T), 0, s, start, stop, 0, a, *queue);
    } else if (by_count) {
      hipLaunchKernelGGL((select_decode_kernel<E, true, T>), g, dim3(T), 0, s, a, *queue);
    } else {
      hipLaunchKernelGGL((select_decode_kernel<E, false, T>), g, dim3(T), 0, s, a, *queue);
    }
  } else if (start || stop) {  // measurement: the runtime stamps the kernel's own begin and end
    if (by_count)
      hipExtLaunchKernelGGL((select_kernel<E, true, T>), grid, dim3(T), 0, s, start, stop, 0, a);
    else
      hipExtLaunchKernelGGL((select_kernel<E, false, T>), grid, dim3(T), 0, s, start, stop, 0, a);
  } else if (by_count) {
    hipLaunchKernelGGL((select_kernel<E, true, T>), grid, dim3(T), 0, s, a);
  } else {
    hipLaunchKernelGGL((select_kernel<E, false, T>), grid, dim3(T), 0, s, a);
  }
}

}  // namespace


hipError_t launch_select(const CacheView &c, const float *logits, const SelectRule &rule, const SelectOut &out,
                         const Plan &plan, const AttnOut &attn, hipStream_t s, hipEvent_t start, hipEvent_t stop,
                         const float2 *summaries, int sub_stride, const SameLaunchQueue *queue) {
  SelectArgs a;
  a.logits = logits;
  a.summaries = summaries;
  a.sub_stride = sub_stride;
  a.seg_cluster_ptr = c.seg_cluster_ptr;
  a.cluster_sizes = c.cluster_sizes;
  a.cluster_offsets = c.cluster_offsets;
  a.cluster_flags = c.cluster_flags;
  a.n_kv_heads = c.n_kv_heads;
  a.n_q_heads = c.n_q_heads;
  a.group = c.group;
  a.max_k = c.max_clusters_per_seg;
  a.uniform_kc = c.uniform_kc;
  a.p1 = rule.p1;
  a.p2 = rule.p2;
  a.p2_absolute = rule.p2_absolute;
  a.k_retained = rule.k_retained;
  a.k_exact = rule.k_exact;
  const bool bc = rule.by_count != 0;
  a.out = out;
  a.plan = plan;
  a.q = c.q;
  a.k_cache = c.k_cache;
  a.v_cache = c.v_cache;
  a.k_centroids = c.k_centroids;
  a.v_centroids = c.v_centroids;
  a.seg_row_base = c.seg_row_base;
  a.attn_out = attn.out;
  a.lse = attn.lse;
  a.out_is_bf16 = attn.out_is_bf16;
  a.scale_log2 = c.sm_scale * kLog2e;
  const dim3 grid(c.batch * c.n_q_heads);
  if (grid.x == 0) return hipSuccess;
  const int k = c.max_clusters_per_seg;
  QueueArgs qa;
  const QueueArgs *q = nullptr;
  if (queue) {
    if (grid.x > (unsigned)kSameLaunchMaxHeads || !plan.ent_src || !attn.out) return hipErrorInvalidValue;
    qa = QueueArgs{queue->partials, queue->planned, queue->splits, (int32_t)grid.x};
    q = &qa;
  }
  // Workgroup size.  The kernel is bound by instruction issue on its one CU (every phase runs once per wave), so a
  // head gets the fewest threads that still leave it at most 8 logits per thread: 512 threads up to 4096 clusters
  // per segment (32 heads x 2048 clusters: 7.7 us instead of 8.6 us for peaked heads, 13.6 us instead of 22.4 us for
  // flat ones), 1024 threads above that (with 16 logits per thread the flat heads lose more than the peaked ones
  // gain).  With more than 512 heads and at most 2048 clusters, 256 threads: four workgroups share a CU instead
  // of running in rounds.
  constexpr int kHalf = kSelThreads / 2, kQuarter = kSelThreads / 4;
  if (grid.x > 512 && k <= 8 * kQuarter) {
    if (k <= 2 * kQuarter) launch_select_e<2, kQuarter>(a, bc, grid, s, start, stop, q);
    else if (k <= 4 * kQuarter) launch_select_e<4, kQuarter>(a, bc, grid, s, start, stop, q);
    else launch_select_e<8, kQuarter>(a, bc, grid, s, start, stop, q);
  } else if (k <= 8 * kHalf) {
    if (k <= 2 * kHalf) launch_select_e<2, kHalf>(a, bc, grid, s, start, stop, q);
    else if (k <= 4 * kHalf) launch_select_e<4, kHalf>(a, bc, grid, s, start, stop, q);
    else launch_select_e<8, kHalf>(a, bc, grid, s, start, stop, q);
  } else if (k <= 8 * kSelThreads) launch_select_e<8, kSelThreads>(a, bc, grid, s, start, stop, q);
  else if (k <= 16 * kSelThreads) launch_select_e<16, kSelThreads>(a, bc, grid, s, start, stop, q);
  else if (k <= 32 * kSelThreads) launch_select_e<32, kSelThreads>(a, bc, grid, s, start, stop, q);
  else if (k <= 64 * kSelThreads) launch_select_e<64, kSelThreads>(a, bc, grid, s, start, stop, q);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_plan(const CacheView &c, const int32_t *sel_ids, const int32_t *n_exact,
                       const int32_t *n_retained, int32_t *n_exact_tokens, const Plan &plan, const AttnOut &attn,
                       hipStream_t s) {
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
  a.attn_out = attn.out;
  a.lse = attn.lse;
  a.out_is_bf16 = attn.out_is_bf16;
  const dim3 grid(c.batch * c.n_q_heads);
  if (grid.x == 0) return hipSuccess;
  hipLaunchKernelGGL(plan_kernel, grid, dim3(kPlanThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace dp
