// Device-side helpers shared by the gfx950 kernels of the Double-P decode step.
//
// Data layout facts the kernels rely on:
//   * head_dim = 128, bf16: one K / V / centroid row is 256 B = 16 lanes x 16 B,
//     so a 16-lane DPP row owns one cache row and a wave64 covers 4 rows per
//     global_load_dwordx4.  Lane t of the row holds dims [8t, 8t+8).
//   * cross-lane sums inside a 16-lane row use DPP modifiers on v_add_f32
//     (quad_perm, row_half_mirror, row_mirror): no LDS traffic.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dp_kernels.hpp"

namespace dp {

constexpr int kRowBytes = kHeadDim * 2;

// ---------------------------------------------------------------- DPP ----
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

// sum over the 16 lanes of a DPP row; every lane of the row gets the total
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_mov<0xB1>(v);   // quad_perm [1,0,3,2]
  v += dpp_mov<0x4E>(v);   // quad_perm [2,3,0,1]
  v += dpp_mov<0x141>(v);  // row_half_mirror
  v += dpp_mov<0x140>(v);  // row_mirror
  return v;
}

// Value of the lane 16 (32) positions away, i.e. the same column of the neighbouring DPP row (of the other half of
// the wave), through the gfx950 row / half swap instructions: two vector-ALU operations instead of a trip through
// the LDS crossbar.  v_permlane16_swap exchanges the odd rows of its first operand with the even rows of its second,
// v_permlane32_swap the upper half of the first with the lower half of the second.
__device__ __forceinline__ uint32_t xor16_u32(uint32_t v) {
  const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
  return (threadIdx.x & 16) ? r[0] : r[1];
}
__device__ __forceinline__ uint32_t xor32_u32(uint32_t v) {
  const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return (threadIdx.x & 32) ? r[0] : r[1];
}
__device__ __forceinline__ float xor16(float v) { return __uint_as_float(xor16_u32(__float_as_uint(v))); }
__device__ __forceinline__ float xor32(float v) { return __uint_as_float(xor32_u32(__float_as_uint(v))); }

// ------------------------------------------------------------- bf16 ------
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

__device__ __forceinline__ void unpack8(const uint4 &r, float (&f)[8]) {
  f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x);
  f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
  f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z);
  f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
}

// fp32 -> bf16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

// 16-byte slice `lane16` of bf16 row `row` of a [rows,128] matrix
__device__ __forceinline__ uint4 load_row_slice(const void *base, int64_t row, int lane16) {
  const char *p = static_cast<const char *>(base) + row * kRowBytes + lane16 * 16;
  return *reinterpret_cast<const uint4 *>(p);
}

// bf16 x bf16 dot product of the lane's 8 dims, accumulated in fp32 by v_dot2c_f32_bf16
// (two multiply-adds per instruction, operands stay packed: no unpacking)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot8_bf16(const uint4 &a, const uint4 &b) {
  float s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.x), __builtin_bit_cast(bf16x2_t, b.x), 0.f, false);
  s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.y), __builtin_bit_cast(bf16x2_t, b.y), s, false);
  s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.z), __builtin_bit_cast(bf16x2_t, b.z), s, false);
  s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.w), __builtin_bit_cast(bf16x2_t, b.w), s, false);
  return s;
}

// partial dot of the lane's 8 dims
__device__ __forceinline__ float dot8(const float (&a)[8], const float (&b)[8]) {
  float s = a[0] * b[0];
#pragma unroll
  for (int i = 1; i < 8; ++i) s = fmaf(a[i], b[i], s);
  return s;
}

// ------------------------------------------- order-preserving float key --
// a > b (as floats, -0 canonicalised to +0 by the caller)  <=>  key(a) > key(b)
__device__ __forceinline__ uint32_t ordered_key(float f) {
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
constexpr uint32_t kKeyLowestFinite = 0x00800000u;  // every finite float has a key >= this; key(-inf) is below

// A workgroup barrier that orders LDS accesses only: unlike __syncthreads() it does not wait for the wave's
// outstanding global memory operations (a counter update in flight, loads issued ahead).
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Marks a kernel argument (a uniform value) as used here: the compiler otherwise fetches an argument that is first
// needed at the end of a kernel (an output pointer, a stride) from the argument segment right there, one more
// dependent round trip behind the last loads.
template <class V>
__device__ __forceinline__ void fetch_early(V v) {
  asm volatile("" ::"s"(v));
}

// ------------------------------------------------- wave / block scans ----
__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

template <typename T>
__device__ __forceinline__ T wave_incl_scan(T v) {
  const int lane = lane_id();
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    T o = __shfl_up(v, d, 64);
    if (lane >= d) v += o;
  }
  return v;
}

// Wave reductions: 4 DPP steps inside each 16-lane row, then 2 cross-row exchanges.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_mov_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
template <int CTRL>
__device__ __forceinline__ unsigned long long dpp_mov_u64(unsigned long long v) {
  const uint32_t lo = dpp_mov_u32<CTRL>((uint32_t)v), hi = dpp_mov_u32<CTRL>((uint32_t)(v >> 32));
  return ((unsigned long long)hi << 32) | lo;
}

// After the 4 DPP steps every lane of a 16-lane row holds its row's result; the four rows are then combined
// through readlane (lanes 0, 16, 32, 48 -> scalar registers), which is much shorter than two cross-row
// shuffles through the LDS crossbar.  The combination order (r0 . r1) . (r2 . r3) is what the shuffles
// gave every lane, so float results keep their bits.
__device__ __forceinline__ uint32_t lane_u32(uint32_t v, int lane) { return (uint32_t)__builtin_amdgcn_readlane((int)v, lane); }
__device__ __forceinline__ unsigned long long lane_u64(unsigned long long v, int lane) {
  return ((unsigned long long)lane_u32((uint32_t)(v >> 32), lane) << 32) | lane_u32((uint32_t)v, lane);
}
__device__ __forceinline__ float lane_f32(float v, int lane) { return __uint_as_float(lane_u32(__float_as_uint(v), lane)); }

__device__ __forceinline__ unsigned long long wave_sum(unsigned long long v) {
  v += dpp_mov_u64<0xB1>(v);
  v += dpp_mov_u64<0x4E>(v);
  v += dpp_mov_u64<0x141>(v);
  v += dpp_mov_u64<0x140>(v);
  return (lane_u64(v, 0) + lane_u64(v, 16)) + (lane_u64(v, 32) + lane_u64(v, 48));
}

__device__ __forceinline__ unsigned long long wave_max(unsigned long long v) {
  auto mx = [](unsigned long long a, unsigned long long b) { return a > b ? a : b; };
  v = mx(v, dpp_mov_u64<0xB1>(v));
  v = mx(v, dpp_mov_u64<0x4E>(v));
  v = mx(v, dpp_mov_u64<0x141>(v));
  v = mx(v, dpp_mov_u64<0x140>(v));
  return mx(mx(lane_u64(v, 0), lane_u64(v, 16)), mx(lane_u64(v, 32), lane_u64(v, 48)));
}

__device__ __forceinline__ int wave_sum(int v) {
  v += (int)dpp_mov_u32<0xB1>((uint32_t)v);
  v += (int)dpp_mov_u32<0x4E>((uint32_t)v);
  v += (int)dpp_mov_u32<0x141>((uint32_t)v);
  v += (int)dpp_mov_u32<0x140>((uint32_t)v);
  return (int)((lane_u32((uint32_t)v, 0) + lane_u32((uint32_t)v, 16)) + (lane_u32((uint32_t)v, 32) + lane_u32((uint32_t)v, 48)));
}

__device__ __forceinline__ float wave_sum(float v) {
  v = row16_sum(v);
  return (lane_f32(v, 0) + lane_f32(v, 16)) + (lane_f32(v, 32) + lane_f32(v, 48));
}

__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_mov<0xB1>(v));
  v = fmaxf(v, dpp_mov<0x4E>(v));
  v = fmaxf(v, dpp_mov<0x141>(v));
  v = fmaxf(v, dpp_mov<0x140>(v));
  return fmaxf(fmaxf(lane_f32(v, 0), lane_f32(v, 16)), fmaxf(lane_f32(v, 32), lane_f32(v, 48)));
}

// Inclusive wave scans of integers: a shift-and-add scan inside each 16-lane row with DPP row shifts (a lane
// without a source reads 0), then the totals of the rows before (lanes 15, 31, 47, through readlane) are added.
__device__ __forceinline__ int wave_incl_scan(int v) {
  v += (int)dpp_mov_u32<0x111>((uint32_t)v);  // row_shr:1
  v += (int)dpp_mov_u32<0x112>((uint32_t)v);  // row_shr:2
  v += (int)dpp_mov_u32<0x114>((uint32_t)v);  // row_shr:4
  v += (int)dpp_mov_u32<0x118>((uint32_t)v);  // row_shr:8
  const int t0 = (int)lane_u32((uint32_t)v, 15), t1 = (int)lane_u32((uint32_t)v, 31), t2 = (int)lane_u32((uint32_t)v, 47);
  const int row = lane_id() >> 4;
  return v + (row == 0 ? 0 : row == 1 ? t0 : row == 2 ? t0 + t1 : t0 + t1 + t2);
}
__device__ __forceinline__ unsigned long long wave_incl_scan(unsigned long long v) {
  v += dpp_mov_u64<0x111>(v);
  v += dpp_mov_u64<0x112>(v);
  v += dpp_mov_u64<0x114>(v);
  v += dpp_mov_u64<0x118>(v);
  const unsigned long long t0 = lane_u64(v, 15), t1 = lane_u64(v, 31), t2 = lane_u64(v, 47);
  const int row = lane_id() >> 4;
  return v + (row == 0 ? 0ull : row == 1 ? t0 : row == 2 ? t0 + t1 : t0 + t1 + t2);
}

// ---- combining the per-wave partials of a block reduction ----
// Lane t of every 16-lane row reads partial t % 16 (one LDS instruction per wave) and the row reduces the 16
// values with DPP steps: every lane ends with the block's result.  Reading all NW partials in every thread costs
// NW LDS instructions per wave, and the one LDS unit of a CU serialises them over the 16 waves of a big workgroup.
__device__ __forceinline__ int row16_sum(int v) {
  v += (int)dpp_mov_u32<0xB1>((uint32_t)v);
  v += (int)dpp_mov_u32<0x4E>((uint32_t)v);
  v += (int)dpp_mov_u32<0x141>((uint32_t)v);
  v += (int)dpp_mov_u32<0x140>((uint32_t)v);
  return v;
}
__device__ __forceinline__ unsigned long long row16_sum(unsigned long long v) {
  v += dpp_mov_u64<0xB1>(v);
  v += dpp_mov_u64<0x4E>(v);
  v += dpp_mov_u64<0x141>(v);
  v += dpp_mov_u64<0x140>(v);
  return v;
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp_mov<0xB1>(v));
  v = fmaxf(v, dpp_mov<0x4E>(v));
  v = fmaxf(v, dpp_mov<0x141>(v));
  v = fmaxf(v, dpp_mov<0x140>(v));
  return v;
}
__device__ __forceinline__ unsigned long long row16_max(unsigned long long v) {
  auto mx = [](unsigned long long a, unsigned long long b) { return a > b ? a : b; };
  v = mx(v, dpp_mov_u64<0xB1>(v));
  v = mx(v, dpp_mov_u64<0x4E>(v));
  v = mx(v, dpp_mov_u64<0x141>(v));
  v = mx(v, dpp_mov_u64<0x140>(v));
  return v;
}
// sum of partials[0 .. NW), NW <= 16, in every lane (call after the barrier that publishes them)
template <typename T, int NW>
__device__ __forceinline__ T partials_sum(const T *partials) {
  static_assert(NW <= 16, "one 16-lane row holds the partials");
  const int t = threadIdx.x & 15;
  return row16_sum(t < NW ? partials[t] : T(0));
}

// Exclusive scan over the block (blockDim.x = 64*NW threads, thread order).
// `total` receives the block sum.  scratch: NW + 1 elements of LDS.  Contains
// two barriers; scratch may be reused after the call returns.
template <typename T, int NW>
__device__ __forceinline__ T block_excl_scan(T v, T *scratch, T &total) {
  static_assert(NW <= 16, "one 16-lane row holds the partials");
  T incl = wave_incl_scan(v);
  if (lane_id() == 63) scratch[wave_id()] = incl;
  __syncthreads();
  const int t = threadIdx.x & 15;
  const T s = t < NW ? scratch[t] : T(0);
  const T tot = row16_sum(s);
  const T base = row16_sum(t < wave_id() ? s : T(0));
  __syncthreads();
  total = tot;
  return base + incl - v;
}

template <typename T, int NW>
__device__ __forceinline__ T block_sum(T v, T *scratch) {
  v = wave_sum(v);
  if (lane_id() == 0) scratch[wave_id()] = v;
  __syncthreads();
  const T tot = partials_sum<T, NW>(scratch);
  __syncthreads();
  return tot;
}

template <int NW>
__device__ __forceinline__ float block_max(float v, float *scratch) {
  static_assert(NW <= 16, "one 16-lane row holds the partials");
  v = wave_max(v);
  if (lane_id() == 0) scratch[wave_id()] = v;
  __syncthreads();
  const int t = threadIdx.x & 15;
  const float m = row16_max(t < NW ? scratch[t] : -INFINITY);
  __syncthreads();
  return m;
}

}  // namespace dp
