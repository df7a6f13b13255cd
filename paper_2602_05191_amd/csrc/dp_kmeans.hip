// Assignment step of the k-means clustering that builds the clustered cache at
// prefill (paper Sec. 4.1): every key goes to its nearest centroid,
//   argmin_c |x - c|^2  =  argmax_c ( x . c - |c|^2 / 2 ),
// ties to the lower centroid index.  Together with dp_build_cluster_cache (the
// update step: centroids = cluster means) this is one Lloyd iteration.
//
// The one dense contraction of this library: tokens x centroids x 128 per KV
// segment (2.2 TFLOP per iteration at 8 x 131072 tokens x 8192 centroids), so
// it runs on the matrix cores: v_mfma_f32_16x16x32_bf16, bf16 operands as
// stored, fp32 accumulation.  MFMA-bound; the operands come from cache (a
// segment's centroids are 2 MB).
//
// A wave owns 64 tokens (4 MFMA row tiles, the A operand, held in registers for
// the whole kernel) and walks the segment's centroids 16 at a time (the B
// operand, loaded from global memory in operand layout, next tile in flight).
// Operand layout of the instruction: lane l holds row l % 16 and the 8
// consecutive k of block l / 16; the result tile holds, in lane l, column
// l % 16 and rows 4 (l / 16) .. + 3.  The accumulator starts at -|c|^2 / 2 of
// the lane's centroid column, so a result element IS the score.  Every lane
// keeps the running best (score, centroid) of its 16 (token, column class)
// pairs: no cross-lane work inside the loop; the 16 column classes of a token
// are merged once at the end (DPP row reduction, lower index wins a tie).
#include "dp_device.hpp"
#include "dp_kernels.hpp"

namespace dp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kKmThreads = 256;
constexpr int kKmTM = 4;                               // 16-token row tiles per wave
constexpr int kKmTokensPerWave = 16 * kKmTM;
constexpr int kKmTokensPerBlock = kKmTokensPerWave * (kKmThreads / 64);

struct KmArgs {
  const void *k_tokens, *centroids;
  const int64_t *seg_row_base;
  const int32_t *seg_rows, *seg_cluster_ptr;
  float *half_norm;      // [total_clusters]
  int32_t *assignment;   // [total_rows]
  float *best_score;     // nullable
  int32_t max_rows, total_clusters;
};

// half_norm[c] = |c|^2 / 2 in fp32; one 16-lane DPP row per centroid
__global__ __launch_bounds__(256) void km_norm_kernel(KmArgs a) {
  const int c = blockIdx.x * 16 + (threadIdx.x >> 4), lane16 = threadIdx.x & 15;
  if (c >= a.total_clusters) return;
  float f[8];
  unpack8(load_row_slice(a.centroids, c, lane16), f);
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s = fmaf(f[i], f[i], s);
  s = row16_sum(s);
  if (lane16 == 0) a.half_norm[c] = 0.5f * s;
}

// 16 B of row `row` at dims [32 j + 8 kq, + 8): the operand slice of lane (row % 16, kq) for k-step j
__device__ __forceinline__ uint4 operand_slice(const void *base, int64_t row, int j, int kq) {
  return *reinterpret_cast<const uint4 *>(static_cast<const char *>(base) + row * kRowBytes + j * 64 + kq * 16);
}

__global__ __launch_bounds__(kKmThreads) void km_assign_kernel(KmArgs a) {
  const int seg = blockIdx.y;
  const int n = min(a.seg_rows[seg], a.max_rows);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int t0 = blockIdx.x * kKmTokensPerBlock + wave * kKmTokensPerWave;  // first token of this wave
  if (t0 >= n) return;
  const int c0 = a.seg_cluster_ptr[seg], kc = a.seg_cluster_ptr[seg + 1] - c0;
  const int64_t r0 = a.seg_row_base[seg];
  const int r = lane & 15, kq = lane >> 4;

  // A operand: token t0 + 16 tm + r; tokens beyond the segment are zero rows (their result is not stored)
  uint4 A[kKmTM][4];
#pragma unroll
  for (int tm = 0; tm < kKmTM; ++tm) {
    const int t = t0 + 16 * tm + r;
#pragma unroll
    for (int j = 0; j < 4; ++j) A[tm][j] = t < n ? operand_slice(a.k_tokens, r0 + t, j, kq) : make_uint4(0, 0, 0, 0);
  }
  // lane's running best for tokens t0 + 16 tm + 4 kq + i among the centroids of column class r
  float best[kKmTM][4];
  int bidx[kKmTM][4];
#pragma unroll
  for (int tm = 0; tm < kKmTM; ++tm)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      best[tm][i] = -INFINITY;
      bidx[tm][i] = 0x7fffffff;
    }

  auto load_tile = [&](int tile, uint4 (&B)[4], float &hn) {
    const int c = tile * 16 + r;  // this lane's centroid column
    if (c < kc) {
#pragma unroll
      for (int j = 0; j < 4; ++j) B[j] = operand_slice(a.centroids, c0 + c, j, kq);
      hn = a.half_norm[c0 + c];
    } else {  // past the segment's centroids: a column that can never win
#pragma unroll
      for (int j = 0; j < 4; ++j) B[j] = make_uint4(0, 0, 0, 0);
      hn = INFINITY;
    }
  };

  const int n_tiles = (kc + 15) / 16;
  uint4 B[4], Bn[4];
  float hn, hnn;
  if (n_tiles > 0) load_tile(0, B, hn);
  for (int tile = 0; tile < n_tiles; ++tile) {
    if (tile + 1 < n_tiles) load_tile(tile + 1, Bn, hnn);
    const int c = tile * 16 + r;
#pragma unroll
    for (int tm = 0; tm < kKmTM; ++tm) {
      f32x4 acc = {-hn, -hn, -hn, -hn};
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, A[tm][j]), __builtin_bit_cast(bf16x8, B[j]),
                                                      acc, 0, 0, 0);
#pragma unroll
      for (int i = 0; i < 4; ++i) {  // centroids come in ascending order: a strict comparison keeps the lowest index
        const bool better = acc[i] > best[tm][i];
        best[tm][i] = better ? acc[i] : best[tm][i];
        bidx[tm][i] = better ? c : bidx[tm][i];
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) B[j] = Bn[j];
    hn = hnn;
  }

  // merge the 16 column classes of each token: max score, lower index on a tie (DPP row exchange)
#pragma unroll
  for (int tm = 0; tm < kKmTM; ++tm)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float s = best[tm][i];
      int id = bidx[tm][i];
      auto step = [&](float os, int oid) {
        const bool take = os > s || (os == s && oid < id);
        s = take ? os : s;
        id = take ? oid : id;
      };
      step(dpp_mov<0xB1>(s), (int)dpp_mov_u32<0xB1>((uint32_t)id));
      step(dpp_mov<0x4E>(s), (int)dpp_mov_u32<0x4E>((uint32_t)id));
      step(dpp_mov<0x141>(s), (int)dpp_mov_u32<0x141>((uint32_t)id));
      step(dpp_mov<0x140>(s), (int)dpp_mov_u32<0x140>((uint32_t)id));
      const int t = t0 + 16 * tm + 4 * kq + i;
      if (r == 0 && t < n) {
        a.assignment[r0 + t] = kc > 0 ? id : -1;
        if (a.best_score) a.best_score[r0 + t] = s;
      }
    }
}

}  // namespace

hipError_t launch_kmeans_assign(const KmeansProblem &p, float *half_norm, hipStream_t s) {
  if (p.n_seg == 0 || p.max_rows == 0) return hipSuccess;
  KmArgs a;
  a.k_tokens = p.k_tokens;
  a.centroids = p.centroids;
  a.seg_row_base = p.seg_row_base;
  a.seg_rows = p.seg_rows;
  a.seg_cluster_ptr = p.seg_cluster_ptr;
  a.half_norm = half_norm;
  a.assignment = p.assignment;
  a.best_score = p.best_score;
  a.max_rows = p.max_rows;
  a.total_clusters = p.total_clusters;
  if (p.total_clusters > 0)
    hipLaunchKernelGGL(km_norm_kernel, dim3((p.total_clusters + 15) / 16), dim3(256), 0, s, a);
  hipLaunchKernelGGL(km_assign_kernel, dim3((p.max_rows + kKmTokensPerBlock - 1) / kKmTokensPerBlock, p.n_seg),
                     dim3(kKmThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace dp
