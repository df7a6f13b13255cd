// Dense decode attention over every token of a KV segment (paper Sec. 2.1,
// Eq. 1): the full-attention baseline that the paper's efficiency figures are
// measured against (Sec. 5.3).
//
// HBM-bound streaming kernel.  The K and V rows of a segment are contiguous, so
// a workgroup streams a row range [split * c, split * c + c) once and scores each
// row against ALL query heads of the GQA group from registers: the cache is
// read once per KV head, not once per query head (512 B per token).  As in the
// sparse kernels a 16-lane DPP row owns one cache row per load (16 B per lane),
// the dot products are packed bf16 dot instructions summed with DPP adds, and
// each DPP row keeps one online-softmax state per head in base-2 form.  The
// per-split partials (m, l, acc[128]) are merged by a second small kernel: no
// counters, no atomics.
#include "dp_attend.hpp"
#include "dp_device.hpp"
#include "dp_kernels.hpp"

namespace dp {
namespace {

constexpr int kDenseThreads = 256;
constexpr int kDenseWaves = kDenseThreads / 64;
constexpr int kDenseGroups = kDenseThreads / 16;
constexpr int kDenseBatch = 4;  // cache rows in flight per DPP row
constexpr int kPartialStride = kHeadDim + 2;

struct DenseArgs {
  const void *q, *k_cache, *v_cache;
  const int64_t *seg_row_base;
  const int32_t *seg_rows;
  float *partials;  // [nh, splits, kPartialStride]
  int32_t n_kv_heads, n_q_heads, group;
  int32_t head0;  // this launch serves heads [head0, head0 + GH) of every group
  int32_t splits, rows_per_split, max_rows;
  float scale_log2;
};

template <int GH>
__global__ __launch_bounds__(kDenseThreads) void dense_kernel(DenseArgs a) {
  __shared__ float s_m[GH][kDenseWaves], s_l[GH][kDenseWaves];
  __shared__ float s_acc[GH][kDenseWaves][kHeadDim];
  const int seg = blockIdx.y, split = blockIdx.x;
  const int R = min(a.seg_rows[seg], a.max_rows);
  const int ra = split * a.rows_per_split;
  const int rb = min(R, ra + a.rows_per_split);
  if (ra >= rb) return;  // the merge kernel derives the number of live splits from R as well

  const int tid = threadIdx.x, lane16 = tid & 15, grp = tid >> 4;
  const int b = seg / a.n_kv_heads, g = seg % a.n_kv_heads;
  const int64_t head_first = (int64_t)b * a.n_q_heads + g * a.group + a.head0;
  const int64_t row0 = a.seg_row_base[seg];

  uint4 qv[GH];
  RowState st[GH];
#pragma unroll
  for (int j = 0; j < GH; ++j) {
    qv[j] = load_row_slice(a.q, head_first + j, lane16);
    row_state_init(st[j]);
  }

  // The 16 DPP rows take consecutive 4-row pieces: one step of the workgroup reads 64 consecutive rows.
  // The loads of the next step are issued before the arithmetic of the current one.
  auto load_piece = [&](int r, uint4 (&kr)[kDenseBatch], uint4 (&vr)[kDenseBatch]) {
#pragma unroll
    for (int u = 0; u < kDenseBatch; ++u) {
      if (r + u < rb) {
        kr[u] = load_row_slice(a.k_cache, row0 + r + u, lane16);
        vr[u] = load_row_slice(a.v_cache, row0 + r + u, lane16);
      } else {
        kr[u] = make_uint4(0, 0, 0, 0);
        vr[u] = make_uint4(0, 0, 0, 0);
      }
    }
  };
  uint4 kraw[kDenseBatch], vraw[kDenseBatch];
  int r = ra + grp * kDenseBatch;
  load_piece(r, kraw, vraw);  // r >= rb loads nothing
  while (r < rb) {
    const int rn = r + kDenseGroups * kDenseBatch;
    uint4 knext[kDenseBatch], vnext[kDenseBatch];
    load_piece(rn, knext, vnext);
    float p[GH][kDenseBatch];
#pragma unroll
    for (int j = 0; j < GH; ++j) {
      float m_new = st[j].m;
#pragma unroll
      for (int u = 0; u < kDenseBatch; ++u) {
        const float d = row16_sum(dot8_bf16(qv[j], kraw[u])) * a.scale_log2;
        p[j][u] = (r + u < rb) ? d : -INFINITY;
        m_new = fmaxf(m_new, p[j][u]);
      }
      // m_new is finite: row r is valid
      const float alpha = exp2f(st[j].m - m_new);
      float lsum = 0.f;
#pragma unroll
      for (int u = 0; u < kDenseBatch; ++u) {
        p[j][u] = exp2f(p[j][u] - m_new);
        lsum += p[j][u];
      }
      st[j].l = st[j].l * alpha + lsum;
#pragma unroll
      for (int i = 0; i < 8; ++i) st[j].acc[i] *= alpha;
      st[j].m = m_new;
    }
#pragma unroll
    for (int u = 0; u < kDenseBatch; ++u) {
      float vf[8];
      unpack8(vraw[u], vf);
#pragma unroll
      for (int j = 0; j < GH; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) st[j].acc[i] = fmaf(p[j][u], vf[i], st[j].acc[i]);
    }
#pragma unroll
    for (int u = 0; u < kDenseBatch; ++u) {
      kraw[u] = knext[u];
      vraw[u] = vnext[u];
    }
    r = rn;
  }

  // merge the DPP rows of each wave, then the waves through LDS
  const int lane = lane_id(), w = wave_id();
#pragma unroll
  for (int j = 0; j < GH; ++j) {
    wave_merge(st[j]);
    if (lane < 16) {
      if (lane == 0) {
        s_m[j][w] = st[j].m;
        s_l[j][w] = st[j].l;
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) s_acc[j][w][lane * 8 + i] = st[j].acc[i];
    }
  }
  __syncthreads();
  // thread t: dim t % 128 of heads t / 128, t / 128 + 2, ...
  for (int j = tid / kHeadDim; j < GH; j += kDenseThreads / kHeadDim) {
    const int t = tid % kHeadDim;
    float M = -INFINITY, L = 0.f, o = 0.f;
#pragma unroll
    for (int v = 0; v < kDenseWaves; ++v) M = fmaxf(M, s_m[j][v]);
#pragma unroll
    for (int v = 0; v < kDenseWaves; ++v) {
      const float wg = (s_m[j][v] == -INFINITY) ? 0.f : exp2f(s_m[j][v] - M);
      L += s_l[j][v] * wg;
      o += s_acc[j][v][t] * wg;
    }
    float *P = a.partials + ((head_first + j) * a.splits + split) * kPartialStride;
    if (t == 0) {
      P[0] = M;
      P[1] = L;
    }
    P[2 + t] = o;
  }
}

struct DenseMergeArgs {
  const float *partials;
  const int32_t *seg_rows;
  void *out;
  float *lse;  // nullable
  int32_t n_kv_heads, n_q_heads, group, splits, rows_per_split, max_rows, out_is_bf16;
};

__global__ __launch_bounds__(kHeadDim) void dense_merge_kernel(DenseMergeArgs a) {
  const int head = blockIdx.x, t = threadIdx.x;
  const int b = head / a.n_q_heads, h = head % a.n_q_heads;
  const int seg = b * a.n_kv_heads + h / a.group;
  const int R = min(a.seg_rows[seg], a.max_rows);
  const int n_active = (R + a.rows_per_split - 1) / a.rows_per_split;
  if (n_active <= 0) {  // an empty segment: zero output
    store_out(a.out, a.out_is_bf16, head, t, 0.f);
    if (a.lse && t == 0) a.lse[head] = -INFINITY;
    return;
  }
  const float *P = a.partials + (int64_t)head * a.splits * kPartialStride;
  float Mx = -INFINITY, Ls = 0.f, os = 0.f;
  for (int s0 = 0; s0 < n_active; s0 += 8) {
    float ms[8], ll[8], oo[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const float *Q = P + min(s0 + u, n_active - 1) * kPartialStride;
      ms[u] = Q[0];
      ll[u] = Q[1];
      oo[u] = Q[2 + t];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (s0 + u < n_active) {  // every live split has at least one row: its m is finite
        const float Mn = fmaxf(Mx, ms[u]);
        const float sc = exp2f(Mx - Mn), wgt = exp2f(ms[u] - Mn);
        Ls = Ls * sc + ll[u] * wgt;
        os = os * sc + oo[u] * wgt;
        Mx = Mn;
      }
    }
  }
  store_out(a.out, a.out_is_bf16, head, t, os / Ls);
  if (a.lse && t == 0) a.lse[head] = (Mx + log2f(Ls)) * kLn2;
}

template <int GH>
void launch_dense_pass(const DenseArgs &a, dim3 grid, hipStream_t s) {
  hipLaunchKernelGGL(dense_kernel<GH>, grid, dim3(kDenseThreads), 0, s, a);
}

}  // namespace

// Equal row ranges stream at equal speed, so the grid is ONE round of workgroups: as many as are resident
// at once (the waves per SIMD that the kernel's registers allow for the widest pass x 256 CUs), each with at
// least 256 rows.  More, shorter workgroups measured 25 % slower (a second, partly idle round).
void dense_split(int max_rows, int n_seg, int group, int max_splits, int *splits, int *rows_per_split) {
  const int resident = group >= 8 ? 512 : group >= 4 ? 768 : group >= 2 ? 1024 : 1280;
  long want = resident / n_seg;
  if (want > max_splits) want = max_splits;
  const long by_rows = ((long)max_rows + 255) / 256;
  if (want > by_rows) want = by_rows;
  if (want < 1) want = 1;
  const long c = kChunkRows * (((long)max_rows + kChunkRows * want - 1) / (kChunkRows * want));
  *rows_per_split = (int)(c > 0 ? c : kChunkRows);
  *splits = (int)(((long)max_rows + *rows_per_split - 1) / *rows_per_split);
  if (*splits < 1) *splits = 1;
}

hipError_t launch_dense(const CacheView &c, const int32_t *seg_rows, float *partials, int max_splits,
                        const AttnOut &attn, hipStream_t s) {
  const int n_seg = c.batch * c.n_kv_heads, nh = c.batch * c.n_q_heads;
  if (nh == 0) return hipSuccess;
  int splits, rows_per_split;
  dense_split(c.max_rows_per_seg, n_seg, c.group, max_splits, &splits, &rows_per_split);
  if (c.max_rows_per_seg > 0) {
    DenseArgs a;
    a.q = c.q;
    a.k_cache = c.k_cache;
    a.v_cache = c.v_cache;
    a.seg_row_base = c.seg_row_base;
    a.seg_rows = seg_rows;
    a.partials = partials;
    a.n_kv_heads = c.n_kv_heads;
    a.n_q_heads = c.n_q_heads;
    a.group = c.group;
    a.splits = splits;
    a.rows_per_split = rows_per_split;
    a.max_rows = c.max_rows_per_seg;
    a.scale_log2 = c.sm_scale * kLog2e;
    const dim3 grid(splits, n_seg);
    // heads of a group are served 8/4/2/1 at a time (one pass over the cache when G is 1, 2, 4 or 8)
    int h0 = 0;
    while (h0 < c.group) {
      const int left = c.group - h0;
      const int gh = left >= 8 ? 8 : left >= 4 ? 4 : left >= 2 ? 2 : 1;
      a.head0 = h0;
      switch (gh) {
        case 8: launch_dense_pass<8>(a, grid, s); break;
        case 4: launch_dense_pass<4>(a, grid, s); break;
        case 2: launch_dense_pass<2>(a, grid, s); break;
        default: launch_dense_pass<1>(a, grid, s); break;
      }
      h0 += gh;
    }
  }
  DenseMergeArgs m;
  m.partials = partials;
  m.seg_rows = seg_rows;
  m.out = attn.out;
  m.lse = attn.lse;
  m.n_kv_heads = c.n_kv_heads;
  m.n_q_heads = c.n_q_heads;
  m.group = c.group;
  m.splits = splits;
  m.rows_per_split = rows_per_split;
  m.max_rows = c.max_rows_per_seg;
  m.out_is_bf16 = attn.out_is_bf16;
  hipLaunchKernelGGL(dense_merge_kernel, dim3(nh), dim3(kHeadDim), 0, s, m);
  return hipGetLastError();
}

}  // namespace dp
