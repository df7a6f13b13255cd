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
// and the 16 states are merged through LDS.  Partials (m, l, acc[128]) go to
// the workspace; a second small kernel merges the splits (log-sum-exp merge),
// normalises and writes the output.
#include "dp_device.hpp"
#include "dp_kernels.hpp"

namespace dp {
namespace {

constexpr int kDecThreads = 256;
constexpr int kDecGroups = kDecThreads / 16;   // 16 DPP rows per workgroup
constexpr int kDecBatch = 4;                   // cache rows in flight per DPP row
constexpr int kDecBlockRows = 256;             // rows resolved per LDS staging round
constexpr int kPartialStride = kHeadDim + 2;   // m, l, acc[128]
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct DecodeArgs {
  const void *q, *k_cache, *v_cache, *k_centroids, *v_centroids;
  const int64_t *seg_row_base;
  const int32_t *seg_cluster_ptr, *cluster_sizes;
  const int32_t *n_exact, *n_retained;
  Plan plan;
  float *partials;
  int32_t n_kv_heads, n_q_heads, group, max_k, splits;
  float scale_log2;  // sm_scale * log2(e)
};

// rows per split of a head with R rows (multiple of kChunkRows)
__device__ __forceinline__ int rows_per_split(int R, int S) {
  return kChunkRows * ((R + kChunkRows * S - 1) / (kChunkRows * S));
}

__global__ __launch_bounds__(kDecThreads) void decode_kernel(DecodeArgs a) {
  __shared__ int s_start[kDecBlockRows + 1];
  __shared__ int s_src[kDecBlockRows + 1];
  __shared__ float s_m[kDecGroups], s_l[kDecGroups];
  __shared__ float s_acc[kDecGroups][kHeadDim];

  const int head = blockIdx.y, split = blockIdx.x;
  const int R = a.plan.head_rows[head];
  if (R <= 0) return;
  const int c = rows_per_split(R, a.splits);
  const int row_a = split * c;
  if (row_a >= R) return;
  const int row_b = min(R, row_a + c);

  const int b = head / a.n_q_heads, h = head % a.n_q_heads;
  const int seg = b * a.n_kv_heads + h / a.group;
  const int c0 = a.seg_cluster_ptr[seg];
  const int64_t seg_row0 = a.seg_row_base[seg];
  const int n_ex = a.n_exact[head], n_rt = a.n_retained[head];
  const int32_t *ent_src = a.plan.ent_src + (int64_t)head * a.max_k;
  const int32_t *row_start = a.plan.row_start + (int64_t)head * (a.max_k + 1);
  const int tid = threadIdx.x, lane16 = tid & 15, grp = tid >> 4;

  float qf[8];
  unpack8(load_row_slice(a.q, (int64_t)head, lane16), qf);
#pragma unroll
  for (int i = 0; i < 8; ++i) qf[i] *= a.scale_log2;

  // online-softmax state of this DPP row, exponents in base 2
  float m_run = -INFINITY, l_run = 0.f, acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;

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

    for (int rb = r0 + grp * kDecBatch; rb < r1; rb += kDecGroups * kDecBatch) {
      // resolve rows rb .. rb+3 : lanes 0..3 of the DPP row search, then broadcast
      int64_t my_row = -1;   // row index in k_cache/v_cache, or in the centroid matrices
      int my_kind = 0;       // 0 invalid, 1 token, 2 centroid pseudo-token
      float my_bias = 0.f;
      if (lane16 < kDecBatch) {
        const int r = rb + lane16;
        if (r < r1) {
          int lo = 0, hi = n_ent;  // largest k in [0, n_ent) with s_start[k] <= r
          while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (s_start[mid] <= r) lo = mid; else hi = mid;
          }
          const int j = ent0 + lo;
          if (j < n_ex) {
            my_kind = 1;
            my_row = seg_row0 + s_src[lo] + (r - s_start[lo]);
          } else {
            my_kind = 2;
            my_row = (int64_t)c0 + s_src[lo];
            my_bias = log2f((float)a.cluster_sizes[c0 + s_src[lo]]);
          }
        }
      }
      uint4 kraw[kDecBatch], vraw[kDecBatch];
      float bias[kDecBatch];
      int kind[kDecBatch];
#pragma unroll
      for (int k = 0; k < kDecBatch; ++k) {
        const int src_lane = (tid & ~15) + k;
        kind[k] = __shfl(my_kind, src_lane, 64);
        const int64_t row = __shfl(my_row, src_lane, 64);
        bias[k] = __shfl(my_bias, src_lane, 64);
        if (kind[k] == 1) {
          kraw[k] = load_row_slice(a.k_cache, row, lane16);
          vraw[k] = load_row_slice(a.v_cache, row, lane16);
        } else if (kind[k] == 2) {
          kraw[k] = load_row_slice(a.k_centroids, row, lane16);
          vraw[k] = load_row_slice(a.v_centroids, row, lane16);
        } else {
          kraw[k] = make_uint4(0, 0, 0, 0);
          vraw[k] = make_uint4(0, 0, 0, 0);
        }
      }
      float x[kDecBatch];
      float m_new = m_run;
#pragma unroll
      for (int k = 0; k < kDecBatch; ++k) {
        float kf[8];
        unpack8(kraw[k], kf);
        const float d = row16_sum(dot8(qf, kf));
        x[k] = kind[k] ? d + bias[k] : -INFINITY;
        m_new = fmaxf(m_new, x[k]);
      }
      if (m_new != -INFINITY) {
        const float alpha = exp2f(m_run - m_new);  // m_run = -inf gives 0
        l_run *= alpha;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] *= alpha;
#pragma unroll
        for (int k = 0; k < kDecBatch; ++k) {
          const float p = exp2f(x[k] - m_new);
          float vf[8];
          unpack8(vraw[k], vf);
          l_run += p;
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[i] = fmaf(p, vf[i], acc[i]);
        }
        m_run = m_new;
      }
    }
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

  // merge the 16 DPP-row states
  if (lane16 == 0) {
    s_m[grp] = m_run;
    s_l[grp] = l_run;
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) s_acc[grp][lane16 * 8 + i] = acc[i];
  __syncthreads();
  if (tid < kHeadDim) {
    float M = s_m[0];
#pragma unroll
    for (int g2 = 1; g2 < kDecGroups; ++g2) M = fmaxf(M, s_m[g2]);
    float L = 0.f, o = 0.f;
#pragma unroll
    for (int g2 = 0; g2 < kDecGroups; ++g2) {
      const float w = (s_m[g2] == -INFINITY) ? 0.f : exp2f(s_m[g2] - M);
      L += s_l[g2] * w;
      o += s_acc[g2][tid] * w;
    }
    float *P = a.partials + ((int64_t)head * a.splits + split) * kPartialStride;
    if (tid == 0) {
      P[0] = M;
      P[1] = L;
    }
    P[2 + tid] = o;
  }
}

struct CombineArgs {
  const int32_t *head_rows;
  const float *partials;
  void *out;
  float *lse;  // nullable
  int32_t splits, out_is_bf16;
};

__global__ __launch_bounds__(kHeadDim) void combine_kernel(CombineArgs a) {
  const int head = blockIdx.x, t = threadIdx.x;
  const int R = a.head_rows[head];
  float o = 0.f, lse = -INFINITY;
  if (R > 0) {
    const int c = rows_per_split(R, a.splits);
    const int n = (R + c - 1) / c;
    const float *P = a.partials + (int64_t)head * a.splits * kPartialStride;
    float M = -INFINITY;
    for (int s = 0; s < n; ++s) M = fmaxf(M, P[s * kPartialStride]);
    float L = 0.f;
    for (int s = 0; s < n; ++s) {
      const float ms = P[s * kPartialStride];
      const float w = (ms == -INFINITY) ? 0.f : exp2f(ms - M);
      L += P[s * kPartialStride + 1] * w;
      o += P[s * kPartialStride + 2 + t] * w;
    }
    o /= L;
    lse = (M + log2f(L)) * kLn2;
  }
  if (a.out_is_bf16)
    static_cast<uint16_t *>(a.out)[(int64_t)head * kHeadDim + t] = (uint16_t)f32_to_bf16_rne(o);
  else
    static_cast<float *>(a.out)[(int64_t)head * kHeadDim + t] = o;
  if (a.lse && t == 0) a.lse[head] = lse;
}

}  // namespace

hipError_t launch_decode(const CacheView &c, const int32_t *n_exact, const int32_t *n_retained, const Plan &plan,
                         float *partials, int splits, void *out, int out_is_bf16, float *lse, hipStream_t s) {
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
  a.n_kv_heads = c.n_kv_heads;
  a.n_q_heads = c.n_q_heads;
  a.group = c.group;
  a.max_k = c.max_clusters_per_seg;
  a.splits = splits;
  a.scale_log2 = c.sm_scale * kLog2e;
  hipLaunchKernelGGL(decode_kernel, dim3(splits, nh), dim3(kDecThreads), 0, s, a);
  CombineArgs cb;
  cb.head_rows = plan.head_rows;
  cb.partials = partials;
  cb.out = out;
  cb.lse = lse;
  cb.splits = splits;
  cb.out_is_bf16 = out_is_bf16;
  hipLaunchKernelGGL(combine_kernel, dim3(nh), dim3(kHeadDim), 0, s, cb);
  return hipGetLastError();
}

}  // namespace dp
