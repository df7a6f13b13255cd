// Stage 1: size-weighted centroid scoring (paper Sec. 4.2, Eq. 3 and Eq. 5):
//   logit[h][i] = sm_scale * (q_h . C_i) + ln s_i
// for every cluster i of a KV segment and every query head h of its GQA group.
//
// HBM-bound streaming kernel: the key-centroid matrix is read exactly once
// (256 B per cluster) and each row is scored against all G query heads of the
// group from registers.  A 16-lane DPP row owns one centroid row (16 B per
// lane, global_load_dwordx4); each lane's 8 products are accumulated by the
// packed bf16 dot instruction and the 16 partial dots are summed with DPP adds.
// Algorithmic traffic per cluster: 256 B centroid + 4 B size read, 4*G B written.
#include <hip/hip_ext.h>

#include "dp_device.hpp"
#include "dp_kernels.hpp"

namespace dp {
namespace {

constexpr int kScoreThreads = 256;                   // 16 DPP rows
#ifndef DP_SCORE_RB
#define DP_SCORE_RB 4
#endif
constexpr int kScoreRowsPerGroup = DP_SCORE_RB;      // centroid rows in flight per 16-lane row
constexpr int kScoreTile = (kScoreThreads / 16) * kScoreRowsPerGroup;  // clusters per workgroup

struct ScoreArgs {
  const void *q, *k_centroids;
  const int32_t *seg_cluster_ptr, *cluster_sizes;
  float *logits;
  int32_t n_kv_heads, n_q_heads, group;
  int32_t head0;       // this launch scores heads [head0, head0 + GH) of each group
  int32_t uniform_kc;  // > 0: every segment has exactly this many clusters
  float sm_scale;
  int32_t *zero_words;  // nullable: n_zero words cleared by the first workgroup (counters of the step's later kernels)
  int32_t n_zero;
};

template <int GH>
__global__ __launch_bounds__(kScoreThreads) void score_kernel(ScoreArgs a) {
  const int seg = blockIdx.y;
  if (a.zero_words && blockIdx.x == 0 && blockIdx.y == 0 && (int)threadIdx.x < a.n_zero) a.zero_words[threadIdx.x] = 0;
  int c0, kc;
  if (a.uniform_kc > 0) {  // no CSR lookup in front of the centroid loads
    c0 = seg * a.uniform_kc;
    kc = a.uniform_kc;
  } else {
    c0 = a.seg_cluster_ptr[seg];
    kc = a.seg_cluster_ptr[seg + 1] - c0;
  }
  const int tile0 = blockIdx.x * kScoreTile;
  if (tile0 >= kc) return;

  const int lane16 = threadIdx.x & 15;
  const int grp = threadIdx.x >> 4;
  const int b = seg / a.n_kv_heads, g = seg % a.n_kv_heads;

  // issue the centroid loads first: this group owns rows tile0 + grp*RB .. +RB-1
  const int i0 = tile0 + grp * kScoreRowsPerGroup;
  uint4 raw[kScoreRowsPerGroup];
  int size[kScoreRowsPerGroup];
#pragma unroll
  for (int k = 0; k < kScoreRowsPerGroup; ++k)
    raw[k] = (i0 + k < kc) ? load_row_slice(a.k_centroids, (int64_t)(c0 + i0 + k), lane16) : make_uint4(0, 0, 0, 0);
  // sizes: one dword per row, the same address for the 16 lanes of the group (a broadcast load; wider
  // or masked loads of the four sizes measured slower)
#pragma unroll
  for (int k = 0; k < kScoreRowsPerGroup; ++k) size[k] = (i0 + k < kc) ? a.cluster_sizes[c0 + i0 + k] : 0;

  // the group's query slices stay packed bf16
  uint4 qv[GH];
#pragma unroll
  for (int j = 0; j < GH; ++j)
    qv[j] = load_row_slice(a.q, (int64_t)b * a.n_q_heads + g * a.group + a.head0 + j, lane16);

  // lane j of the group ends up with head j's logits of the group's RB consecutive clusters
  float mine[kScoreRowsPerGroup];
#pragma unroll
  for (int k = 0; k < kScoreRowsPerGroup; ++k) {
    mine[k] = 0.f;
#pragma unroll
    for (int j = 0; j < GH; ++j) {
      const float d = row16_sum(dot8_bf16(qv[j], raw[k]));
      if (lane16 == j) mine[k] = d;
    }
  }
  if (lane16 < GH && i0 < kc) {
    float *out = a.logits + (int64_t)a.group * c0 + (int64_t)(a.head0 + lane16) * kc + i0;
    float v[kScoreRowsPerGroup];
#pragma unroll
    for (int k = 0; k < kScoreRowsPerGroup; ++k) {
      // ln s from the hardware log2 (1 ulp), exact for s = 1
      v[k] = (size[k] > 0) ? fmaf(mine[k], a.sm_scale, __builtin_amdgcn_logf((float)size[k]) * 0.6931471805599453f)
                           : -INFINITY;
    }
    if (kScoreRowsPerGroup == 4 && i0 + 3 < kc && (reinterpret_cast<uintptr_t>(out) & 15) == 0) {
      *reinterpret_cast<float4 *>(out) = make_float4(v[0], v[1 % kScoreRowsPerGroup], v[2 % kScoreRowsPerGroup],
                                                     v[3 % kScoreRowsPerGroup]);
    } else {
#pragma unroll
      for (int k = 0; k < kScoreRowsPerGroup; ++k)
        if (i0 + k < kc) out[k] = v[k];
    }
  }
}

}  // namespace

template <int GH>
void launch_one(const ScoreArgs &a, dim3 grid, hipStream_t s, hipEvent_t start, hipEvent_t stop) {
  if (start || stop)
    hipExtLaunchKernelGGL(score_kernel<GH>, grid, dim3(kScoreThreads), 0, s, start, stop, 0, a);
  else
    hipLaunchKernelGGL(score_kernel<GH>, grid, dim3(kScoreThreads), 0, s, a);
}

hipError_t launch_score(const CacheView &c, float *logits, hipStream_t s, hipEvent_t start, hipEvent_t stop,
                        int32_t *zero_words, int n_zero) {
  ScoreArgs a;
  a.q = c.q;
  a.k_centroids = c.k_centroids;
  a.seg_cluster_ptr = c.seg_cluster_ptr;
  a.cluster_sizes = c.cluster_sizes;
  a.logits = logits;
  a.n_kv_heads = c.n_kv_heads;
  a.n_q_heads = c.n_q_heads;
  a.group = c.group;
  a.sm_scale = c.sm_scale;
  a.uniform_kc = c.uniform_kc;
  a.zero_words = n_zero <= kScoreThreads ? zero_words : nullptr;
  a.n_zero = n_zero;
  const dim3 grid((c.max_clusters_per_seg + kScoreTile - 1) / kScoreTile, c.batch * c.n_kv_heads);
  if (grid.x == 0 || grid.y == 0) return hipSuccess;
  // heads of a group are scored 8/4/2/1 at a time (one pass when G is 1, 2, 4 or 8)
  int h0 = 0;
  while (h0 < c.group) {
    const int left = c.group - h0;
    const int gh = left >= 8 ? 8 : left >= 4 ? 4 : left >= 2 ? 2 : 1;
    a.head0 = h0;
    if (h0 > 0) a.zero_words = nullptr;  // cleared once, by the first pass
    // with several passes the events bracket the first pass's begin and the last pass's end
    hipEvent_t ev0 = (h0 == 0) ? start : nullptr, ev1 = (h0 + gh >= c.group) ? stop : nullptr;
    switch (gh) {
      case 8: launch_one<8>(a, grid, s, ev0, ev1); break;
      case 4: launch_one<4>(a, grid, s, ev0, ev1); break;
      case 2: launch_one<2>(a, grid, s, ev0, ev1); break;
      default: launch_one<1>(a, grid, s, ev0, ev1); break;
    }
    h0 += gh;
  }
  return hipGetLastError();
}

}  // namespace dp
