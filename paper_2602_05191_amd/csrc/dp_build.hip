// Prefill side of the clustered cache (paper Sec. 4.1, Eq. 2): from K / V in
// token order and one cluster id per token, build what the decode step reads:
// the cluster-contiguous K / V rows, per-cluster sizes and offsets, the key
// centroids C_i (mean key) and the value aggregates V^Sigma_i and V-bar_i.
//
// A stable counting sort by cluster id with the segmented mean taken while the
// rows move.  HBM-bound: every K / V row is read once (a 256 B run at its token's
// place) and written once (clusters are written as contiguous runs); nothing
// is read back.  Everything is deterministic: counts are integers, a token's
// place inside its cluster is its token order, and the means are fp64 sums
// taken in row order and rounded once to bf16.
//
//   rank     per 1024-token block: the block's count of every cluster (integer
//            atomics on a table in LDS, written out as one row) and a token's
//            rank among the EARLIER tokens of its block with the same id: 0 when
//            the token is alone with its id in the block (the common case), else
//            by pairwise compare among the tokens that are not
//   scan     per cluster: exclusive prefix of those counts over the blocks
//            (in place) and the cluster's size
//   offsets  per segment: exclusive prefix of the sizes
//   place    row of a token = offset of its cluster + count of its cluster in
//            earlier blocks + rank; written per token (token_row) and, inverted,
//            per row (the token that fills it)
//   gather   one 16-lane row per cluster walks the cluster's rows in order:
//            fetches each row's token, stores it in place and adds it to the sums
// The update step of k-means (mean key of every cluster, nothing moved) is the same
// sequence with the cache pointers left null.
#include "dp_device.hpp"
#include "dp_kernels.hpp"

namespace dp {
namespace {

constexpr int kBuildBlock = 1024;  // tokens per block = threads per workgroup of rank / scatter

struct BuildArgs {
  const void *k_tokens, *v_tokens;
  const int32_t *assignment;
  const int64_t *seg_row_base;
  const int32_t *seg_rows, *seg_cluster_ptr;
  void *k_cache, *v_cache, *k_centroids, *v_centroids;
  int32_t *cluster_offsets, *cluster_sizes, *token_row;  // token_row nullable
  float *v_sums;                                         // nullable
  int32_t *hist;                                         // [n_seg, n_blocks, max_kc]
  uint16_t *rank;                                        // [n_seg, n_blocks * kBuildBlock]
  int32_t *row_token;                                    // [n_seg, max_rows]: segment-relative token of each cache row
  int32_t n_blocks, max_kc, max_rows;
};

__global__ __launch_bounds__(kBuildBlock) void build_rank_kernel(BuildArgs a) {
  extern __shared__ uint32_t s_count[];  // two 16-bit counts per word: clusters 2 w and 2 w + 1 (a count is <= 1024)
  __shared__ int s_id[kBuildBlock];      // ids of the tokens that share their cluster inside the block, in token order
  __shared__ int s_scr[kBuildBlock / 64 + 1];
  const int seg = blockIdx.y, blk = blockIdx.x, tid = threadIdx.x;
  const int n = min(a.seg_rows[seg], a.max_rows);
  if (blk * kBuildBlock >= n) return;
  const int c0 = a.seg_cluster_ptr[seg], kc = min(a.seg_cluster_ptr[seg + 1] - c0, a.max_kc);
  const int t = blk * kBuildBlock + tid;
  for (int w = tid; 2 * w < kc; w += kBuildBlock) s_count[w] = 0;
  int c = -1;
  if (t < n) {
    c = a.assignment[a.seg_row_base[seg] + t];
    if ((unsigned)c >= (unsigned)kc) c = -1;  // a token without a valid cluster is left out
  }
  __syncthreads();
  if (c >= 0) atomicAdd(&s_count[c >> 1], 1u << (16 * (c & 1)));  // integer counts: any order gives the same table
  __syncthreads();
  int32_t *row = a.hist + ((size_t)seg * a.n_blocks + blk) * a.max_kc;
  for (int i = tid; i < kc; i += kBuildBlock) row[i] = (int32_t)((s_count[i >> 1] >> (16 * (i & 1))) & 0xffffu);
  const bool shared_id = c >= 0 && ((s_count[c >> 1] >> (16 * (c & 1))) & 0xffffu) > 1u;
  int m;
  const int pos = block_excl_scan<int, kBuildBlock / 64>(shared_id ? 1 : 0, s_scr, m);
  if (shared_id) s_id[pos] = c;
  __syncthreads();
  if (c < 0) return;
  int earlier = 0;
  if (shared_id)  // the list is in token order: the earlier tokens are its first pos entries
    for (int j = 0; j < pos; ++j) earlier += s_id[j] == c;
  a.rank[((size_t)seg * a.n_blocks + blk) * kBuildBlock + tid] = (uint16_t)earlier;
}

__global__ __launch_bounds__(256) void build_scan_kernel(BuildArgs a) {
  const int seg = blockIdx.y;
  const int c0 = a.seg_cluster_ptr[seg], kc = min(a.seg_cluster_ptr[seg + 1] - c0, a.max_kc);
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= kc) return;
  const int n = min(a.seg_rows[seg], a.max_rows);
  const int blocks = (n + kBuildBlock - 1) / kBuildBlock;
  int32_t *h = a.hist + (size_t)seg * a.n_blocks * a.max_kc + c;
  int run = 0;
  for (int b0 = 0; b0 < blocks; b0 += 8) {  // 8 independent loads in flight, then the running prefix
    int v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = (b0 + u < blocks) ? h[(size_t)(b0 + u) * a.max_kc] : 0;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (b0 + u < blocks) h[(size_t)(b0 + u) * a.max_kc] = run;
      run += v[u];
    }
  }
  a.cluster_sizes[c0 + c] = run;
}

__global__ __launch_bounds__(1024) void build_offsets_kernel(BuildArgs a) {
  __shared__ int scr[1024 / 64 + 1];
  const int seg = blockIdx.x, tid = threadIdx.x;
  const int c0 = a.seg_cluster_ptr[seg], kc = a.seg_cluster_ptr[seg + 1] - c0;
  int carry = 0;
  for (int i0 = 0; i0 < kc; i0 += 1024) {
    const int i = i0 + tid;
    // clusters beyond the host's bound received no size: they are reported empty
    const int s = (i < kc && i < a.max_kc) ? a.cluster_sizes[c0 + i] : 0;
    int tot;
    const int ex = block_excl_scan<int, 1024 / 64>(s, scr, tot);
    if (i < kc) {
      a.cluster_offsets[c0 + i] = carry + ex;
      if (i >= a.max_kc) a.cluster_sizes[c0 + i] = 0;
    }
    carry += tot;
  }
}

__global__ __launch_bounds__(256) void build_place_kernel(BuildArgs a) {
  const int seg = blockIdx.y;
  const int n = min(a.seg_rows[seg], a.max_rows);
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t >= n) return;
  const int c0 = a.seg_cluster_ptr[seg], kc = min(a.seg_cluster_ptr[seg + 1] - c0, a.max_kc);
  const int64_t r0 = a.seg_row_base[seg];
  const int blk = t / kBuildBlock;
  const int c = a.assignment[r0 + t];
  int dest = -1;
  if ((unsigned)c < (unsigned)kc) {
    dest = a.cluster_offsets[c0 + c] + a.hist[((size_t)seg * a.n_blocks + blk) * a.max_kc + c] +
           a.rank[(size_t)seg * a.n_blocks * kBuildBlock + t];
    a.row_token[(size_t)seg * a.max_rows + dest] = t;
  }
  if (a.token_row) a.token_row[r0 + t] = dest;
}

// double -> bf16 bits with ONE rounding to 8 significant bits, ties to even.  Values whose magnitude
// is below the bf16 normal range go through float (two roundings, irrelevant at 1e-38).
__device__ __forceinline__ uint32_t f64_to_bf16_rne(double x) {
  const unsigned long long u = (unsigned long long)__double_as_longlong(x);
  const int e = (int)((u >> 52) & 0x7ff) - 1023 + 127;  // bf16 / float exponent field
  if (e <= 0 || e >= 255) return f32_to_bf16_rne((float)x);
  const unsigned long long man = u & 0xfffffffffffffull;
  unsigned long long top = man >> 45;                   // 7 explicit mantissa bits
  const unsigned long long rest = man & ((1ull << 45) - 1), half = 1ull << 44;
  uint32_t bits = ((uint32_t)(u >> 63) << 15) | ((uint32_t)e << 7) | (uint32_t)top;
  if (rest > half || (rest == half && (top & 1))) bits += 1;  // a carry runs into the exponent, as it should
  return bits;
}

// kMove = false: keys only (the update step of k-means): nothing is moved, no value is read, a cluster without
// tokens keeps the centroid it has, and four times as many key rows are in flight (a cluster's rows are summed in
// order by one 16-lane row, so a very large cluster is a chain of dependent rounds of loads).
template <bool kMove>
__global__ __launch_bounds__(256) void build_gather_kernel(BuildArgs a) {
  const int seg = blockIdx.y;
  const int c0 = a.seg_cluster_ptr[seg], kc = a.seg_cluster_ptr[seg + 1] - c0;
  const int lane16 = threadIdx.x & 15, grp = threadIdx.x >> 4;
  const int ci = blockIdx.x * 16 + grp;
  if (ci >= kc) return;
  const int s = a.cluster_sizes[c0 + ci];
  const int off = a.cluster_offsets[c0 + ci];
  const int64_t r0 = a.seg_row_base[seg], row0 = r0 + off;
  const int32_t *tok = a.row_token + (size_t)seg * a.max_rows + off;
  constexpr bool move = kMove;
  if (!move && s == 0) return;
  double ks[8], vs[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) ks[i] = vs[i] = 0.0;
  constexpr int kB = kMove ? 4 : 16;  // rows in flight per 16-lane row
  for (int rb = 0; rb < s; rb += 16) {
    // the tokens of the next 16 rows of the cluster, one per lane of the 16-lane row
    const int mine = rb + lane16 < s ? tok[rb + lane16] : 0;
    const int nb = min(16, s - rb);
    for (int r = 0; r < nb; r += kB) {
      uint4 kr[kB], vr[kB];
#pragma unroll
      for (int u = 0; u < kB; ++u) {
        const int t = __shfl(mine, r + u, 16);
        kr[u] = make_uint4(0, 0, 0, 0);
        vr[u] = make_uint4(0, 0, 0, 0);
        if (r + u < nb) {
          kr[u] = load_row_slice(a.k_tokens, r0 + t, lane16);
          if (move) vr[u] = load_row_slice(a.v_tokens, r0 + t, lane16);
        }
      }
#pragma unroll
      for (int u = 0; u < kB; ++u) {  // rows beyond the cluster add +0.0: the sums are unchanged
        if (move && r + u < nb) {
          const int64_t row = row0 + rb + r + u;
          *reinterpret_cast<uint4 *>(static_cast<char *>(a.k_cache) + row * kRowBytes + lane16 * 16) = kr[u];
          *reinterpret_cast<uint4 *>(static_cast<char *>(a.v_cache) + row * kRowBytes + lane16 * 16) = vr[u];
        }
        float kf[8], vf[8];
        unpack8(kr[u], kf);
        unpack8(vr[u], vf);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          ks[i] += (double)kf[i];
          vs[i] += (double)vf[i];
        }
      }
    }
  }
  uint32_t kb[8], vb[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    kb[i] = s > 0 ? f64_to_bf16_rne(ks[i] / (double)s) : 0u;
    vb[i] = s > 0 ? f64_to_bf16_rne(vs[i] / (double)s) : 0u;
  }
  const size_t o16 = (size_t)(c0 + ci) * kRowBytes + lane16 * 16;
  *reinterpret_cast<uint4 *>(static_cast<char *>(a.k_centroids) + o16) =
      make_uint4(kb[0] | (kb[1] << 16), kb[2] | (kb[3] << 16), kb[4] | (kb[5] << 16), kb[6] | (kb[7] << 16));
  if (!move) return;
  *reinterpret_cast<uint4 *>(static_cast<char *>(a.v_centroids) + o16) =
      make_uint4(vb[0] | (vb[1] << 16), vb[2] | (vb[3] << 16), vb[4] | (vb[5] << 16), vb[6] | (vb[7] << 16));
  if (a.v_sums) {
    float *o = a.v_sums + (size_t)(c0 + ci) * kHeadDim + lane16 * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (float)vs[i];
  }
}

}  // namespace

void build_workspace_layout(int n_seg, int max_rows, int max_kc, size_t *hist_bytes, size_t *rank_bytes,
                            size_t *row_token_bytes, int *n_blocks) {
  const int nb = (max_rows + kBuildBlock - 1) / kBuildBlock;
  *n_blocks = nb;
  *hist_bytes = ((size_t)n_seg * nb * max_kc * sizeof(int32_t) + 255) / 256 * 256;
  *rank_bytes = ((size_t)n_seg * nb * kBuildBlock * sizeof(uint16_t) + 255) / 256 * 256;
  *row_token_bytes = ((size_t)n_seg * max_rows * sizeof(int32_t) + 255) / 256 * 256;
}

hipError_t launch_build(const BuildProblem &p, void *workspace, hipStream_t s) {
  if (p.n_seg == 0) return hipSuccess;
  size_t hist_bytes, rank_bytes, row_token_bytes;
  int n_blocks;
  build_workspace_layout(p.n_seg, p.max_rows, p.max_kc, &hist_bytes, &rank_bytes, &row_token_bytes, &n_blocks);
  BuildArgs a;
  a.k_tokens = p.k_tokens;
  a.v_tokens = p.v_tokens;
  a.assignment = p.assignment;
  a.seg_row_base = p.seg_row_base;
  a.seg_rows = p.seg_rows;
  a.seg_cluster_ptr = p.seg_cluster_ptr;
  a.k_cache = p.k_cache;
  a.v_cache = p.v_cache;
  a.k_centroids = p.k_centroids;
  a.v_centroids = p.v_centroids;
  a.cluster_offsets = p.cluster_offsets;
  a.cluster_sizes = p.cluster_sizes;
  a.token_row = p.token_row;
  a.v_sums = p.v_sums;
  a.hist = static_cast<int32_t *>(workspace);
  a.rank = reinterpret_cast<uint16_t *>(static_cast<char *>(workspace) + hist_bytes);
  a.row_token = reinterpret_cast<int32_t *>(static_cast<char *>(workspace) + hist_bytes + rank_bytes);
  a.n_blocks = n_blocks;
  a.max_kc = p.max_kc;
  a.max_rows = p.max_rows;
  if (n_blocks > 0 && p.max_kc > 0) {
    // the count table of a block lives in LDS: 2 bytes per cluster of the longest segment (128 KB at the 65536 limit)
    const size_t lds = ((size_t)p.max_kc + 1) / 2 * sizeof(uint32_t);
    if (lds > 32768) {
      const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(build_rank_kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(build_rank_kernel, dim3(n_blocks, p.n_seg), dim3(kBuildBlock), lds, s, a);
  }
  if (p.max_kc > 0)
    hipLaunchKernelGGL(build_scan_kernel, dim3((p.max_kc + 255) / 256, p.n_seg), dim3(256), 0, s, a);
  hipLaunchKernelGGL(build_offsets_kernel, dim3(p.n_seg), dim3(1024), 0, s, a);
  if (n_blocks > 0 && p.max_kc > 0)
    hipLaunchKernelGGL(build_place_kernel, dim3((p.max_rows + 255) / 256, p.n_seg), dim3(256), 0, s, a);
  if (p.max_kc > 0) {
    const dim3 grid((p.max_kc + 15) / 16, p.n_seg);
    if (p.k_cache) hipLaunchKernelGGL(build_gather_kernel<true>, grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL(build_gather_kernel<false>, grid, dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace dp
