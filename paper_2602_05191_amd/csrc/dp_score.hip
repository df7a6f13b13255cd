// Stage 1: size-weighted centroid scoring (paper Sec. 4.2, Eq. 3 and Eq. 5):
//   logit[h][i] = sm_scale * (q_h . C_i) + ln s_i
// for every cluster i of a KV segment and every query head h of its GQA group.
//
// HBM-bound streaming kernels: the key-centroid matrix is read exactly once
// (256 B per cluster) and each row is scored against all G query heads of the
// group at once.  Algorithmic traffic per cluster: 256 B centroid + 4 B size
// read, 4*G B written.  Two formulations, chosen by G:
//   G <= 4  vector ALU: packed bf16 dots (v_dot2c_f32_bf16) and a 16-lane DPP
//           reduction per row and head, 2.25 instructions per cluster and head,
//           behind whole-row loads (every load instruction reads 4 rows of 256 B)
//   G >  4  matrix core: the scores of 16 clusters against up to 16 heads are one
//           [16 x 128] x [128 x 16] contraction, four v_mfma_f32_16x16x32_bf16
//           (64 matrix-core cycles per 16 clusters, whatever G is).  The operands
//           go from global memory straight into the MFMA register layout: lane l
//           loads, for cluster row l % 16, the 16-byte chunks l / 16 + 4 j of the
//           row, so a load instruction reads 64 contiguous bytes of 16 rows and
//           the four together read the rows whole.  Heads beyond the group are
//           zero columns.
// Measured (one MI355X, cold centroids): G = 8, 32 x 8192 clusters: 17.0 us on the
// vector ALU, 15.0 us on the matrix core; G = 4: 8 x 8192 clusters 5.8 vs 5.4 us,
// 128 x 1280 clusters 10.0 vs 10.7 us, 128 ragged segments of 512..2048 clusters
// 12.3 vs 14.5 us (the 64-byte load pattern streams slower over many short
// segments), so G = 4 stays on the vector ALU.
#include <hip/hip_ext.h>

#include "dp_device.hpp"
#include "dp_kernels.hpp"

namespace dp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kScoreThreads = 256;                   // 4 waves
constexpr int kScoreHeads = 16;                      // query heads per pass: the columns of one MFMA tile
constexpr int kScoreTile = (kScoreThreads / 64) * 16;  // clusters per workgroup and tile step: a 16-row MFMA tile per wave
constexpr int kScoreValuMaxGroup = 4;  // groups up to this size are scored on the vector ALU, larger ones on the matrix core
constexpr int kScoreMinWgs = 512;  // a launch keeps at least this many workgroups when it takes several tiles per wave

struct ScoreArgs {
  const void *q, *k_centroids;
  const int32_t *seg_cluster_ptr, *cluster_sizes;
  float *logits;
  int32_t n_kv_heads, n_q_heads, group;
  int32_t head0;       // this launch scores heads [head0, head0 + 16) of each group
  int32_t uniform_kc;  // > 0: every segment has exactly this many clusters
  float sm_scale;
  int32_t *zero_words;  // nullable: n_zero words cleared by the first workgroup of every segment, 256 each (counters of the step's later kernels)
  int32_t n_zero;
  // nullable: per head and sub-tile of kSubTile consecutive clusters, (max logit, sum of exp(logit - max)); row
  // stride sub_stride.  Lets the selection find the top of the distribution without reading every logit.
  float2 *summaries;
  int32_t sub_stride;
};

// Both kernels leave the logits of one head's sub-tile (16 consecutive clusters) in the four lanes l, l ^ 16,
// l ^ 32, l ^ 48 of a wave, four consecutive clusters each (-inf where there is no cluster).  Every lane of the
// wave must call this; `writer` is true in the one lane per head that stores the result.
__device__ __forceinline__ void publish_summary(const float (&v)[4], bool writer, float2 *dst) {
  float m = fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3]));
  m = fmaxf(m, xor16(m));
  m = fmaxf(m, xor32(m));
  float s = 0.f;
  if (m > -INFINITY) {
#pragma unroll
    for (int k = 0; k < 4; ++k) s += __builtin_amdgcn_exp2f((v[k] - m) * 1.4426950408889634f);  // exp2(-inf) = 0
  }
  s += xor16(s);  // fixed order: (row0 + row1) + (row2 + row3) in every lane
  s += xor32(s);
  if (writer) *dst = make_float2(m, s);
}

// The same scores on the vector ALU, for small groups: a 16-lane DPP row owns kValuRows consecutive centroid rows
// (16 B per lane: every load instruction reads 4 whole rows), each lane's 8 products are accumulated by the packed
// bf16 dot instruction and the 16 partial dots are summed with DPP adds.  2.25 vector instructions per cluster and
// head: up to G = 4 they hide behind the loads and the wholly contiguous load pattern streams faster.
constexpr int kValuRows = 4;  // centroid rows in flight per 16-lane row; 16 rows x 4 = the 64 clusters of a workgroup
template <int GH>
__global__ __launch_bounds__(kScoreThreads) void score_valu_kernel(
    const void *k_centroids, const int32_t *cluster_sizes, const void *q,
    const int32_t *__restrict__ seg_ptr, int uniform_kc, int n_kv_heads, int n_q_heads, int group, int head0, ScoreArgs a) {
  const int seg = blockIdx.y;
  if (a.zero_words && blockIdx.x == 0 && (int)(blockIdx.y * kScoreThreads + threadIdx.x) < a.n_zero)
    a.zero_words[blockIdx.y * kScoreThreads + threadIdx.x] = 0;
  int c0, kc;
  if (uniform_kc > 0) {  // no CSR lookup in front of the centroid loads
    c0 = seg * uniform_kc;
    kc = uniform_kc;
  } else {
    // the table comes as a separate restrict parameter: the compiler then reads it with scalar loads (as a member
    // of the argument struct it was a vector load and a wait in front of the centroid loads: 0.8 us on ragged batches)
    c0 = seg_ptr[seg];
    kc = seg_ptr[seg + 1] - c0;
  }
  const int tile0 = blockIdx.x * kScoreTile;  // 64 clusters per workgroup here too
  if (tile0 >= kc) return;

  const int lane16 = threadIdx.x & 15;
  const int grp = threadIdx.x >> 4;
  const int b = seg / n_kv_heads, g = seg % n_kv_heads;

  // issue the centroid loads first: this group owns rows tile0 + grp*RB .. +RB-1
  const int i0 = tile0 + grp * kValuRows;
  uint4 raw[kValuRows];
  int size[kValuRows];
#pragma unroll
  for (int k = 0; k < kValuRows; ++k)
    raw[k] = (i0 + k < kc) ? load_row_slice(k_centroids, (int64_t)(c0 + i0 + k), lane16) : make_uint4(0, 0, 0, 0);
  // sizes: one dword per row, the same address for the 16 lanes of the group (a broadcast load; wider
  // or masked loads of the four sizes measured slower)
#pragma unroll
  for (int k = 0; k < kValuRows; ++k) size[k] = (i0 + k < kc) ? cluster_sizes[c0 + i0 + k] : 0;

  // the group's query slices stay packed bf16
  uint4 qv[GH];
#pragma unroll
  for (int j = 0; j < GH; ++j)
    qv[j] = load_row_slice(q, (int64_t)b * n_q_heads + g * group + head0 + j, lane16);

  // what the end of the kernel needs from the argument segment is fetched while the loads are in flight
  fetch_early(a.logits);
  fetch_early(a.summaries);
  fetch_early(a.sub_stride);
  fetch_early(a.sm_scale);

  // lane j of the group ends up with head j's logits of the group's RB consecutive clusters
  float mine[kValuRows];
#pragma unroll
  for (int k = 0; k < kValuRows; ++k) {
    mine[k] = 0.f;
#pragma unroll
    for (int j = 0; j < GH; ++j) {
      const float d = row16_sum(dot8_bf16(qv[j], raw[k]));
      if (lane16 == j) mine[k] = d;
    }
  }
  float v[kValuRows];
#pragma unroll
  for (int k = 0; k < kValuRows; ++k) {
    // ln s from the hardware log2 (1 ulp), exact for s = 1; a cluster beyond the segment was given size 0
    v[k] = (size[k] > 0) ? fmaf(mine[k], a.sm_scale, __builtin_amdgcn_logf((float)size[k]) * 0.6931471805599453f)
                         : -INFINITY;
  }
  if (a.summaries) {  // a wave's four rows are the 16 consecutive clusters tile0 + 16 w .. + 15
    const int sub0 = tile0 + (threadIdx.x >> 6) * 16;
    const int64_t head = (int64_t)b * n_q_heads + g * group + head0 + lane16;
    publish_summary(v, lane16 < GH && (threadIdx.x & 63) < 16 && sub0 < kc,
                    a.summaries + (lane16 < GH ? head : 0) * a.sub_stride + (sub0 >> 4));
  }
  if (lane16 < GH && i0 < kc) {
    float *out = a.logits + (int64_t)group * c0 + (int64_t)(head0 + lane16) * kc + i0;
    if (kValuRows == 4 && i0 + 3 < kc && (reinterpret_cast<uintptr_t>(out) & 15) == 0) {
      *reinterpret_cast<float4 *>(out) = make_float4(v[0], v[1 % kValuRows], v[2 % kValuRows],
                                                     v[3 % kValuRows]);
    } else {
#pragma unroll
      for (int k = 0; k < kValuRows; ++k)
        if (i0 + k < kc) out[k] = v[k];
    }
  }
}


// (The arguments that the first loads depend on are leading scalar kernel parameters: the compiler flag
// -amdgpu-kernarg-preload-count puts those into registers when a wave is launched, so no argument load sits in front
// of the centroid loads.)
// RT = 16-row tiles per wave.  Every wave loads the group's queries once and all its centroid tiles up front: a
// larger RT means fewer query loads per centroid byte and more bytes in flight per wave, at the price of fewer
// workgroups (measured: 17.4 -> 15.2 us with RT = 4 on 32 segments of 8192 clusters, G = 8; 6.0 -> 5.7 us with
// RT = 2 on 8 segments of 8192 clusters, G = 4).
template <int RT>
__global__ __launch_bounds__(kScoreThreads) void score_kernel(
    const void *k_centroids, const int32_t *cluster_sizes, const void *q,
    const int32_t *__restrict__ seg_ptr, int uniform_kc, int n_kv_heads, int n_q_heads, int group, int head0, ScoreArgs a) {
  const int seg = blockIdx.y;
  if (a.zero_words && blockIdx.x == 0 && (int)(blockIdx.y * kScoreThreads + threadIdx.x) < a.n_zero)
    a.zero_words[blockIdx.y * kScoreThreads + threadIdx.x] = 0;
  int c0, kc;
  if (uniform_kc > 0) {  // no CSR lookup in front of the centroid loads
    c0 = seg * uniform_kc;
    kc = uniform_kc;
  } else {
    c0 = seg_ptr[seg];  // a separate restrict parameter: a scalar load
    kc = seg_ptr[seg + 1] - c0;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 15, kq = lane >> 4;
  // the workgroup's kScoreTile * RT consecutive clusters; tile t of wave w is rows (4 t + w) * 16 .. + 15 of them
  const int base = blockIdx.x * (kScoreTile * RT) + wave * 16;
  if (base >= kc) return;  // no barrier below: a wave may leave alone
  const int b = seg / n_kv_heads, g = seg % n_kv_heads;

  const bool head_live = head0 + r < group;
  // B operand first (its few cache lines are hot, and loads return in issue order: behind the centroid stream the
  // queries cost 0.25 us more): query head r of the pass (a zero column beyond the group), chunks kq + 4 j
  uint4 Q[4];
  {
    const char *row = static_cast<const char *>(q) +
                      ((int64_t)b * n_q_heads + g * group + (head_live ? head0 + r : 0)) * kRowBytes + kq * 16;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      Q[j] = head_live ? *reinterpret_cast<const uint4 *>(row + j * 64) : make_uint4(0, 0, 0, 0);
  }
  // A operand: row r of the tile, the same chunks
  uint4 A[RT][4];
#pragma unroll
  for (int t = 0; t < RT; ++t) {
    const int row = base + t * kScoreTile + r;
    const bool live = row < kc;
    const char *src = static_cast<const char *>(k_centroids) + (int64_t)(c0 + row) * kRowBytes + kq * 16;
#pragma unroll
    for (int j = 0; j < 4; ++j) A[t][j] = live ? *reinterpret_cast<const uint4 *>(src + j * 64) : make_uint4(0, 0, 0, 0);
  }
  // the lane's results are head r of the pass, clusters i0 .. i0 + 3 of each tile; their sizes: one dword each,
  // the same address for the lanes of a group (a broadcast load; wider or masked loads measured slower)
  int size[RT][4];
#pragma unroll
  for (int t = 0; t < RT; ++t) {
    const int i0 = base + t * kScoreTile + 4 * kq;
#pragma unroll
    for (int k = 0; k < 4; ++k) size[t][k] = (i0 + k < kc) ? cluster_sizes[c0 + i0 + k] : 0;
  }
  fetch_early(a.logits);  // the end of the kernel's arguments, fetched while the loads are in flight
  fetch_early(a.summaries);
  fetch_early(a.sub_stride);
  fetch_early(a.sm_scale);
#pragma unroll
  for (int t = 0; t < RT; ++t) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 4; ++j)
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, A[t][j]),
                                                    __builtin_bit_cast(bf16x8, Q[j]), acc, 0, 0, 0);
    const int i0 = base + t * kScoreTile + 4 * kq;
    float v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      // ln s from the hardware log2 (1 ulp), exact for s = 1; a cluster beyond the segment was given size 0
      v[k] = (size[t][k] > 0)
                 ? fmaf(acc[k], a.sm_scale, __builtin_amdgcn_logf((float)size[t][k]) * 0.6931471805599453f)
                 : -INFINITY;
    }
    if (a.summaries) {  // the tile is the 16 consecutive clusters base + 64 t .. + 15
      const int sub0 = base + t * kScoreTile;
      const int64_t head = (int64_t)b * n_q_heads + g * group + head0 + r;
      publish_summary(v, head_live && kq == 0 && sub0 < kc,
                      a.summaries + (head_live ? head : 0) * a.sub_stride + (sub0 >> 4));
    }
    if (head_live && i0 < kc) {
      float *out = a.logits + (int64_t)group * c0 + (int64_t)(head0 + r) * kc + i0;
      if (i0 + 3 < kc && (reinterpret_cast<uintptr_t>(out) & 15) == 0) {
        *reinterpret_cast<float4 *>(out) = make_float4(v[0], v[1], v[2], v[3]);
      } else {
#pragma unroll
        for (int k = 0; k < 4; ++k)
          if (i0 + k < kc) out[k] = v[k];
      }
    }
  }
}

}  // namespace

#define HOT_ARGS(a) (a).k_centroids, (a).cluster_sizes, (a).q, (a).seg_cluster_ptr, (a).uniform_kc, (a).n_kv_heads, (a).n_q_heads, (a).group, (a).head0

template <int GH>
void launch_valu(const ScoreArgs &a, dim3 grid, hipStream_t s, hipEvent_t start, hipEvent_t stop) {
  if (start || stop)
    hipExtLaunchKernelGGL(score_valu_kernel<GH>, grid, dim3(kScoreThreads), 0, s, start, stop, 0, HOT_ARGS(a), a);
  else
    hipLaunchKernelGGL(score_valu_kernel<GH>, grid, dim3(kScoreThreads), 0, s, HOT_ARGS(a), a);
}

template <int RT>
void launch_one(const ScoreArgs &a, dim3 grid, hipStream_t s, hipEvent_t start, hipEvent_t stop) {
  if (start || stop)
    hipExtLaunchKernelGGL(score_kernel<RT>, grid, dim3(kScoreThreads), 0, s, start, stop, 0, HOT_ARGS(a), a);
  else
    hipLaunchKernelGGL(score_kernel<RT>, grid, dim3(kScoreThreads), 0, s, HOT_ARGS(a), a);
}

hipError_t launch_score(const CacheView &c, float *logits, hipStream_t s, hipEvent_t start, hipEvent_t stop,
                        int32_t *zero_words, int n_zero, float2 *summaries, int sub_stride) {
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
  a.zero_words = n_zero <= kScoreThreads * c.batch * c.n_kv_heads ? zero_words : nullptr;  // 256 words per segment
  a.n_zero = n_zero;
  a.summaries = summaries;
  a.sub_stride = sub_stride;
  if (c.max_clusters_per_seg == 0 || c.batch * c.n_kv_heads == 0) return hipSuccess;
  if (c.group <= kScoreValuMaxGroup) {
    // one pass: 4, 2 or 1 heads at a time
    const dim3 vgrid((c.max_clusters_per_seg + kScoreTile - 1) / kScoreTile, c.batch * c.n_kv_heads);
    int h0 = 0;
    while (h0 < c.group) {
      const int left = c.group - h0, gh = left >= 4 ? 4 : left >= 2 ? 2 : 1;
      a.head0 = h0;
      if (h0 > 0) a.zero_words = nullptr;  // cleared once, by the first pass
      hipEvent_t ev0 = (h0 == 0) ? start : nullptr, ev1 = (h0 + gh >= c.group) ? stop : nullptr;
      switch (gh) {
        case 4: launch_valu<4>(a, vgrid, s, ev0, ev1); break;
        case 2: launch_valu<2>(a, vgrid, s, ev0, ev1); break;
        default: launch_valu<1>(a, vgrid, s, ev0, ev1); break;
      }
      h0 += gh;
    }
    return hipGetLastError();
  }
  // tiles per wave: as many (1, 2 or 4) as still leave the launch kScoreMinWgs workgroups
  const int64_t wgs1 = (int64_t)((c.max_clusters_per_seg + kScoreTile - 1) / kScoreTile) * c.batch * c.n_kv_heads;
  const int rt = wgs1 >= 4 * kScoreMinWgs ? 4 : wgs1 >= 2 * kScoreMinWgs ? 2 : 1;
  const dim3 grid((c.max_clusters_per_seg + kScoreTile * rt - 1) / (kScoreTile * rt), c.batch * c.n_kv_heads);
  // the heads of a group are scored 16 at a time (one pass for G <= 16)
  for (int h0 = 0; h0 < c.group; h0 += kScoreHeads) {
    a.head0 = h0;
    if (h0 > 0) a.zero_words = nullptr;  // cleared once, by the first pass
    // with several passes the events bracket the first pass's begin and the last pass's end
    hipEvent_t ev0 = (h0 == 0) ? start : nullptr, ev1 = (h0 + kScoreHeads >= c.group) ? stop : nullptr;
    switch (rt) {
      case 4: launch_one<4>(a, grid, s, ev0, ev1); break;
      case 2: launch_one<2>(a, grid, s, ev0, ev1); break;
      default: launch_one<1>(a, grid, s, ev0, ev1); break;
    }
  }
  return hipGetLastError();
}

}  // namespace dp
