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
// A wave owns 16 x TM tokens (TM MFMA row tiles, the A operand, held in registers
// for the whole kernel).  The workgroup walks the segment's centroids 64 at a time:
// the block is fetched once from global memory by all 256 threads, kept in LDS
// (three blocks in rotation, rows padded to 272 B so that the 16 rows an operand
// read touches fall into different banks) and read from there by the four waves
// as the B operand: the operand read of the next tile is issued before the
// current tile's MFMAs (also across block borders: the next block is already in
// LDS), and the block after that travels global -> registers -> LDS behind them.
// The register budget is held at 168 (three waves per SIMD): with two waves the
// same loop is 20 % slower.
// Operand layout of the instruction: lane l holds row l % 16 and the 8
// consecutive k of block l / 16; the result tile holds, in lane l, column
// l % 16 and rows 4 (l / 16) .. + 3.  The accumulator starts at -|c|^2 / 2 of
// the lane's centroid column, so a result element IS the score.  Every lane
// keeps the running best (score, centroid) of its 4 x TM (token, column class)
// pairs: no cross-lane work inside the loop; the 16 column classes of a token
// are merged once at the end (DPP row reduction, lower index wins a tie).
#include "dp_device.hpp"
#include "dp_kernels.hpp"

namespace dp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kKmThreads = 256;
constexpr int kKmTM = 4;                     // 16-token row tiles per wave
constexpr int kKmTokensPerWave = 16 * kKmTM;
constexpr int kKmTokensPerBlock = kKmTokensPerWave * (kKmThreads / 64);
constexpr int kKmCB = 64;                     // centroids per LDS block (a multiple of 64: 256 threads fetch 64 rows per pass)
constexpr int kKmBufs = 3;                              // LDS blocks in rotation: computed on, next (already stored), being filled
constexpr int kKmRowPad = kRowBytes + 16;              // LDS row stride: 68 words, 4 r mod 64 banks for row r

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

__global__ __launch_bounds__(kKmThreads) __attribute__((amdgpu_waves_per_eu(3, 3))) void km_assign_kernel(KmArgs a) {
  __shared__ __attribute__((aligned(16))) char s_c[kKmBufs][kKmCB * kKmRowPad];
  __shared__ float s_hn[kKmBufs][kKmCB];
  const int seg = blockIdx.y;
  const int n = min(a.seg_rows[seg], a.max_rows);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int blk0 = blockIdx.x * kKmTokensPerBlock;
  if (blk0 >= n) return;  // uniform in the workgroup
  const int t0 = blk0 + wave * kKmTokensPerWave;  // first token of this wave (a wave past the end only helps to load)
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

  // global -> registers -> LDS: per pass of 64 rows, thread tid fetches 64 B (quarter tid & 3) of row tid >> 2
  constexpr int kPasses = kKmCB / 64;
  const int lrow = tid >> 2, lq = tid & 3;
  uint4 stage[kPasses][4];
  float stage_hn[kPasses];
  auto fetch_block = [&](int blk) {
#pragma unroll
    for (int ps = 0; ps < kPasses; ++ps) {
      const int c = blk * kKmCB + ps * 64 + lrow;
      if (c < kc) {
        const char *src = static_cast<const char *>(a.centroids) + (int64_t)(c0 + c) * kRowBytes + lq * 64;
#pragma unroll
        for (int u = 0; u < 4; ++u) stage[ps][u] = *reinterpret_cast<const uint4 *>(src + 16 * u);
        stage_hn[ps] = a.half_norm[c0 + c];
      } else {  // past the segment's centroids: columns that can never win
#pragma unroll
        for (int u = 0; u < 4; ++u) stage[ps][u] = make_uint4(0, 0, 0, 0);
        stage_hn[ps] = INFINITY;
      }
    }
  };
  auto store_block = [&](int buf) {
#pragma unroll
    for (int ps = 0; ps < kPasses; ++ps) {
      char *dst = s_c[buf] + (ps * 64 + lrow) * kKmRowPad + lq * 64;
#pragma unroll
      for (int u = 0; u < 4; ++u) *reinterpret_cast<uint4 *>(dst + 16 * u) = stage[ps][u];
      if (lq == 0) s_hn[buf][ps * 64 + lrow] = stage_hn[ps];
    }
  };

  // B operand of tile tt of LDS block buf, and the lane's -|c|^2/2 start value
  struct Tile {
    uint4 B[4];
    float hn;
  };
  auto read_tile = [&](int buf, int tt) {
    Tile t;
    const char *row = s_c[buf] + (tt * 16 + r) * kKmRowPad + kq * 16;
#pragma unroll
    for (int j = 0; j < 4; ++j) t.B[j] = *reinterpret_cast<const uint4 *>(row + j * 64);
    t.hn = s_hn[buf][tt * 16 + r];
    return t;
  };

  // Three LDS blocks in rotation: block blk is computed on while block blk + 1 (stored one iteration earlier) is
  // already readable, so the operand read of the NEXT tile is always issued before the current tile's MFMAs,
  // across block borders too, and block blk + 2 travels global -> registers -> LDS behind them.
  const int n_blocks = (kc + kKmCB - 1) / kKmCB;
  if (n_blocks > 0) {
    fetch_block(0);
    store_block(0);
  }
  if (n_blocks > 1) {
    fetch_block(1);
    store_block(1);
  }
  __syncthreads();
  Tile next = read_tile(0, 0);  // harmless when there is no block: never used
  int buf = 0;
  for (int blk = 0; blk < n_blocks; ++blk) {
    const int buf1 = buf == kKmBufs - 1 ? 0 : buf + 1, buf2 = buf1 == kKmBufs - 1 ? 0 : buf1 + 1;
    if (blk + 2 < n_blocks) fetch_block(blk + 2);  // in flight during this block's MFMAs
#pragma unroll 1
    for (int tt = 0; tt < kKmCB / 16; ++tt) {
      const Tile cur = next;
      const bool last = tt == kKmCB / 16 - 1;
      next = read_tile(last ? buf1 : buf, last ? 0 : tt + 1);  // past the last block: a stale block, never used
      const int c = blk * kKmCB + tt * 16 + r;  // this lane's centroid column
      // TM independent accumulation chains, advanced together: no MFMA waits for its predecessor
      f32x4 acc[kKmTM];
#pragma unroll
      for (int tm = 0; tm < kKmTM; ++tm) acc[tm] = f32x4{-cur.hn, -cur.hn, -cur.hn, -cur.hn};
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int tm = 0; tm < kKmTM; ++tm)
          acc[tm] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, A[tm][j]),
                                                            __builtin_bit_cast(bf16x8, cur.B[j]), acc[tm], 0, 0, 0);
#pragma unroll
      for (int tm = 0; tm < kKmTM; ++tm)
#pragma unroll
        for (int i = 0; i < 4; ++i) {  // centroids come in ascending order: a strict comparison keeps the lowest index
          const bool better = acc[tm][i] > best[tm][i];
          best[tm][i] = better ? acc[tm][i] : best[tm][i];
          bidx[tm][i] = better ? c : bidx[tm][i];
        }
    }
    // buf2 held block blk - 1, last read before the barrier that ended the previous iteration
    if (blk + 2 < n_blocks) store_block(buf2);
    __syncthreads();
    buf = buf1;
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

// One 16-lane row copies one key row: centroid c of the segment starts as the key of token floor(c * n / kc).
__global__ __launch_bounds__(256) void km_init_strided_kernel(KmArgs a, void *centroids) {
  const int seg = blockIdx.y;
  const int c0 = a.seg_cluster_ptr[seg], kc = a.seg_cluster_ptr[seg + 1] - c0;
  const int lane16 = threadIdx.x & 15, c = blockIdx.x * 16 + (threadIdx.x >> 4);
  if (c >= kc) return;
  const int n = min(a.seg_rows[seg], a.max_rows);
  uint4 row = make_uint4(0, 0, 0, 0);
  if (n > 0) row = load_row_slice(a.k_tokens, a.seg_row_base[seg] + (int64_t)c * n / kc, lane16);
  *reinterpret_cast<uint4 *>(static_cast<char *>(centroids) + (size_t)(c0 + c) * kRowBytes + lane16 * 16) = row;
}

}  // namespace

hipError_t launch_kmeans_init_strided(const KmeansProblem &p, void *centroids, int max_kc, hipStream_t s) {
  if (p.n_seg == 0 || max_kc == 0) return hipSuccess;
  KmArgs a{};
  a.k_tokens = p.k_tokens;
  a.seg_row_base = p.seg_row_base;
  a.seg_rows = p.seg_rows;
  a.seg_cluster_ptr = p.seg_cluster_ptr;
  a.max_rows = p.max_rows;
  hipLaunchKernelGGL(km_init_strided_kernel, dim3((max_kc + 15) / 16, p.n_seg), dim3(256), 0, s, a, centroids);
  return hipGetLastError();
}

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
