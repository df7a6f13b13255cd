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
//   move     a workgroup per 16 clusters walks their rows (one contiguous run) in
//            chunks: fetches each row's token, stores it in place, and sums the
//            chunk's rows column by column from a copy in LDS
// The update step of k-means (mean key of every cluster, nothing moved) is the same
// sequence with the cache pointers left null: the last kernel then fetches keys only and stores no row.
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

// The move.  A workgroup owns 16 consecutive clusters, whose rows are one contiguous run of the cache.  The run is
// taken in chunks of 64 rows: the sixteen 16-lane rows of the workgroup fetch four rows each (whatever the sizes
// of the clusters, every lane has the same number of loads in flight), store them in place and leave a copy in LDS;
// then thread d sums column d (key dimensions, then value dimensions) of the chunk's rows in row order, in fp64, and
// writes a cluster's means when its last row has gone by.  A sum carries over from chunk to chunk.
// kMove = false: keys only (the update step of k-means): nothing is stored in place, no value is read, and a cluster
// without tokens keeps the centroid it has.
constexpr int kMoveRows = 64;

template <bool kMove>
__global__ __launch_bounds__(256) void build_move_kernel(BuildArgs a) {
  __shared__ __align__(16) uint16_t s_rows[kMoveRows][2 * kHeadDim];  // key | value of every row of the chunk
  const int seg = blockIdx.y, tid = threadIdx.x;
  const int c0 = a.seg_cluster_ptr[seg], kc = a.seg_cluster_ptr[seg + 1] - c0;
  const int64_t r0 = a.seg_row_base[seg];
  const int cf = blockIdx.x * 16;
  if (cf >= kc) return;
  const int ncl = min(16, kc - cf);
  const int lane16 = tid & 15, grp = tid >> 4;
  // every 16-lane row holds the bounds of the workgroup's clusters, one per lane
  const int cme = c0 + cf + min(lane16, ncl - 1);
  const int sz = a.cluster_sizes[cme], off = a.cluster_offsets[cme];
  const int run0 = __shfl(off, 0, 16), n_run = __shfl(off + sz, ncl - 1, 16) - run0;
  const int my_end = off + sz - run0;  // where the cluster ends inside the run

  const int32_t *tok = a.row_token + (size_t)seg * a.max_rows + run0;
  // lanes u, u + 4, ... of a 16-lane row: the token of the row's u-th share of the chunk (row 16 u + grp)
  auto token_of = [&](int base) { return tok[min(base + 16 * (lane16 & 3) + grp, n_run - 1)]; };
  auto flush = [&](int c, int s, double sum) {
    if (!kMove && (s == 0 || tid >= kHeadDim)) return;
    const uint32_t bits = s > 0 ? f64_to_bf16_rne(sum / (double)s) : 0u;
    const size_t o = (size_t)(c0 + cf + c) * kHeadDim;
    if (tid < kHeadDim) {
      static_cast<uint16_t *>(a.k_centroids)[o + tid] = (uint16_t)bits;
    } else {
      static_cast<uint16_t *>(a.v_centroids)[o + tid - kHeadDim] = (uint16_t)bits;
      if (a.v_sums) a.v_sums[o + tid - kHeadDim] = (float)sum;
    }
  };

  double acc = 0.0;
  int cur = 0;  // the cluster whose rows are being summed: the same in every thread
  int cur_end = __builtin_amdgcn_readfirstlane(__shfl(my_end, 0, 16));
  int cur_sz = __builtin_amdgcn_readfirstlane(__shfl(sz, 0, 16));
  int mine = n_run > 0 ? token_of(0) : 0;
  for (int base = 0; base < n_run; base += kMoveRows) {
    const int nb = min(kMoveRows, n_run - base);
    uint4 kr[4], vr[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {  // shares beyond the run fetch its last row again and are not stored
      const int t = __shfl(mine, u, 16);
      kr[u] = load_row_slice(a.k_tokens, r0 + t, lane16);
      if (kMove) vr[u] = load_row_slice(a.v_tokens, r0 + t, lane16);
    }
    mine = token_of(base + kMoveRows);  // the next chunk's tokens arrive while this chunk is summed
    lds_barrier();                      // the previous chunk has been summed
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      *reinterpret_cast<uint4 *>(&s_rows[16 * u + grp][lane16 * 8]) = kr[u];
      if (kMove) *reinterpret_cast<uint4 *>(&s_rows[16 * u + grp][kHeadDim + lane16 * 8]) = vr[u];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {  // after the copies: a wait placed behind a store would wait for the store
      const int j = 16 * u + grp;
      if (kMove && j < nb) {
        const int64_t row = r0 + run0 + base + j;
        *reinterpret_cast<uint4 *>(static_cast<char *>(a.k_cache) + row * kRowBytes + lane16 * 16) = kr[u];
        *reinterpret_cast<uint4 *>(static_cast<char *>(a.v_cache) + row * kRowBytes + lane16 * 16) = vr[u];
      }
    }
    lds_barrier();
    int j = 0;
    while (cur < ncl) {
      const int hi = min(cur_end - base, nb);
      if (!kMove && tid >= kHeadDim) j = hi;  // keys only: the upper half of the workgroup has no column
      for (; j + 8 <= hi; j += 8) {
        uint16_t x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) x[u] = s_rows[j + u][tid];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += (double)__uint_as_float((uint32_t)x[u] << 16);
      }
      for (; j < hi; ++j) acc += (double)__uint_as_float((uint32_t)s_rows[j][tid] << 16);
      if (cur_end - base > nb) break;  // the cluster goes on in the next chunk
      flush(cur, cur_sz, acc);
      acc = 0.0;
      ++cur;
      if (cur < ncl) {
        cur_end = __builtin_amdgcn_readfirstlane(__shfl(my_end, cur, 16));
        cur_sz = __builtin_amdgcn_readfirstlane(__shfl(sz, cur, 16));
      }
    }
  }
  for (; cur < ncl; ++cur)  // a workgroup without rows: its clusters are empty
    flush(cur, 0, 0.0);
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
    if (p.k_cache) hipLaunchKernelGGL(build_move_kernel<true>, grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL(build_move_kernel<false>, grid, dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace dp
