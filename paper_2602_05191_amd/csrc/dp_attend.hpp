// Weighted online-softmax attention over a head's row list (paper Eq. 8, Eq. 9),
// shared by the split decode kernel and by the selection kernel's inline path
// for heads with few rows.
//
// Row list of a head: entries j = 0 .. n_rt-1; entry j < n_ex is an exact
// cluster (its s rows are consecutive K/V cache rows, additive weight 0),
// entry j >= n_ex is an approximated cluster (ONE pseudo-row: key centroid,
// mean value, additive weight log2 s).  row_start[j] is the exclusive prefix
// of rows.  A 16-lane DPP row ("group") owns one cache row per load: lane t
// holds dims [8t, 8t+8) of K for the dot product and of V for the accumulation.
// All exponents are base 2 (logits are scaled by sm_scale * log2 e).
#pragma once

#include "dp_device.hpp"

namespace dp {

constexpr int kAttendBatch = 4;  // cache rows in flight per group

struct RowState {
  float m, l, acc[8];
};

__device__ __forceinline__ void row_state_init(RowState &s) {
  s.m = -INFINITY;
  s.l = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s.acc[i] = 0.f;
}

struct RowSources {
  const void *k_cache, *v_cache, *k_centroids, *v_centroids;
  const int32_t *seg_sizes;  // cluster_sizes + c0 of the head's segment
  int64_t seg_row0;          // first cache row of the segment
  int64_t c0;                // first centroid row of the segment
  // A/B variant only (kGathered): the head's exact rows copied to a contiguous buffer, list row r at gather_row0 + r
  const void *k_gather, *v_gather;
  int64_t gather_row0;
};

// Attend rows ra, ra+1, .., ra+B-1, then ra+stride .. (B rows in flight per step), below rb.  s_start[0 .. n_ent] and s_src[0 .. n_ent)
// are the staged row_start / ent_src of entries ent0 .. ent0+n_ent-1, which
// cover [ra, rb) (s_start[0] <= ra).  Every lane of the group runs the same
// entry walk (uniform inside the group), so nothing is exchanged between lanes
// except the DPP sum of the dot product.
template <bool kGathered = false, int B = kAttendBatch>
__device__ __forceinline__ void attend_rows(RowState &st, const uint4 &qv, float scale_log2, const RowSources &src,
                                            const int *s_start, const int *s_src, int n_ent, int ent0, int n_ex,
                                            int ra, int rb, int stride, int lane16) {
  if (ra >= rb) return;
  // entry that holds row ra: largest k in [0, n_ent) with s_start[k] <= ra
  int k = 0;
  {
    int hi = n_ent;
    while (hi - k > 1) {
      const int mid = (k + hi) >> 1;
      if (s_start[mid] <= ra) k = mid; else hi = mid;
    }
  }
  int next_start = s_start[k + 1];
  for (int r = ra; r < rb; r += stride) {
    uint4 kraw[B], vraw[B];
    int ssz[B];  // the row's additive weight is log2 of this: 1 for a token, the cluster's size for a pseudo-token, 0 (-inf) for no row
#pragma unroll
    for (int u = 0; u < B; ++u) {
      const int row = r + u;
      ssz[u] = 0;
      if (row < rb) {
        while (row >= next_start) {  // walk forward to the entry that holds this row
          ++k;
          next_start = s_start[k + 1];
        }
        const int s = s_src[k];
        if (ent0 + k < n_ex) {
          const int64_t g = src.seg_row0 + s + (row - s_start[k]);
          ssz[u] = 1;
          if (kGathered) {
            kraw[u] = load_row_slice(src.k_gather, src.gather_row0 + row, lane16);
            vraw[u] = load_row_slice(src.v_gather, src.gather_row0 + row, lane16);
          } else {
            kraw[u] = load_row_slice(src.k_cache, g, lane16);
            vraw[u] = load_row_slice(src.v_cache, g, lane16);
          }
        } else {
          ssz[u] = src.seg_sizes[s];
          kraw[u] = load_row_slice(src.k_centroids, src.c0 + s, lane16);
          vraw[u] = load_row_slice(src.v_centroids, src.c0 + s, lane16);
        }
      } else {
        kraw[u] = make_uint4(0, 0, 0, 0);
        vraw[u] = make_uint4(0, 0, 0, 0);
      }
    }
    float x[B];
    float m_new = st.m;
#pragma unroll
    for (int u = 0; u < B; ++u) {
      // log2(1) = 0 exactly; log2(0) = -inf: a missing row (its key is zero) weighs nothing
      x[u] = fmaf(row16_sum(dot8_bf16(qv, kraw[u])), scale_log2, log2f((float)ssz[u]));
      m_new = fmaxf(m_new, x[u]);
    }
    // m_new is finite here: row r is valid
    const float alpha = exp2f(st.m - m_new);  // st.m = -inf gives 0
    st.l *= alpha;
#pragma unroll
    for (int i = 0; i < 8; ++i) st.acc[i] *= alpha;
#pragma unroll
    for (int u = 0; u < B; ++u) {
      const float p = exp2f(x[u] - m_new);
      float vf[8];
      unpack8(vraw[u], vf);
      st.l += p;
#pragma unroll
      for (int i = 0; i < 8; ++i) st.acc[i] = fmaf(p, vf[i], st.acc[i]);
    }
    st.m = m_new;
  }
}

// Merge the 4 groups of a wave (log-sum-exp merge); every group ends with the wave's state.
__device__ __forceinline__ void wave_merge(RowState &st) {
#pragma unroll
  for (int d = 16; d <= 32; d <<= 1) {
    const float om = d == 16 ? xor16(st.m) : xor32(st.m);
    const float M = fmaxf(st.m, om);
    const float wa = (st.m == -INFINITY) ? 0.f : exp2f(st.m - M);
    const float wb = (om == -INFINITY) ? 0.f : exp2f(om - M);
    st.l = st.l * wa + (d == 16 ? xor16(st.l) : xor32(st.l)) * wb;
#pragma unroll
    for (int i = 0; i < 8; ++i) st.acc[i] = st.acc[i] * wa + (d == 16 ? xor16(st.acc[i]) : xor32(st.acc[i])) * wb;
    st.m = M;
  }
}

// Merge the first n_waves waves of a workgroup through LDS (the others hold no rows).
// s_m / s_l: NW floats, s_acc: NW x 128 floats.  Returns, for threads tid < 128: M, L and the
// unnormalised output of dim tid.  n_waves is block-uniform, 1 <= n_waves <= NW.
template <int NW>
__device__ __forceinline__ void block_merge(RowState &st, float *s_m, float *s_l, float (*s_acc)[kHeadDim],
                                            int n_waves, float &M, float &L, float &o) {
  const int lane = lane_id(), w = wave_id();
  if (w < n_waves) {
    wave_merge(st);
    if (lane < 16) {
      if (lane == 0) {
        s_m[w] = st.m;
        s_l[w] = st.l;
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) s_acc[w][lane * 8 + i] = st.acc[i];
    }
  }
  lds_barrier();  // only LDS is exchanged here
  M = -INFINITY;
  L = 0.f;
  o = 0.f;
  if (threadIdx.x < kHeadDim) {
    for (int g = 0; g < n_waves; ++g) M = fmaxf(M, s_m[g]);
    for (int g = 0; g < n_waves; ++g) {
      const float wg = (s_m[g] == -INFINITY) ? 0.f : exp2f(s_m[g] - M);
      L += s_l[g] * wg;
      o += s_acc[g][threadIdx.x] * wg;
    }
  }
}

__device__ __forceinline__ void store_out(void *out, int out_is_bf16, int64_t head, int t, float v) {
  if (out_is_bf16)
    static_cast<uint16_t *>(out)[head * kHeadDim + t] = (uint16_t)f32_to_bf16_rne(v);
  else
    static_cast<float *>(out)[head * kHeadDim + t] = v;
}

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

}  // namespace dp
