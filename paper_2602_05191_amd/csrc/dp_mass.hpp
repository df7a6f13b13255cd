// Fixed-point softmax masses and the two top-p thresholds, shared by the
// selection kernel and its sort-based variant so that both take every decision
// on the same integers.
#pragma once

#include "dp_attend.hpp"
#include "dp_device.hpp"

namespace dp {

typedef unsigned long long u64;

constexpr float kCut = 27.72f;  // just under 40 ln 2: beyond it the fixed-point mass is 0

// floor(w * 2^40) for 0 <= w <= 1, exactly, with 32-bit conversions only
__device__ __forceinline__ u64 fixed40(float w) {
  const float t = w * 256.0f;
  const uint32_t hi = (uint32_t)t;
  const uint32_t lo = (uint32_t)((t - (float)hi) * 4294967296.0f);
  return ((u64)hi << 32) | lo;
}

// d = max - logit >= 0 (+inf for an empty cluster)
__device__ __forceinline__ u64 fx_mass(float d) {
  return d < kCut ? fixed40(__builtin_amdgcn_exp2f(-d * kLog2e)) : 0;
}

// first threshold in units of 2^-40: tau1 in [1, W] (Eq. 7 with the inclusive comparison)
__device__ __forceinline__ u64 top_p_first_tau(float p1, u64 W) {
  const u64 t = (u64)ceil((double)p1 * (double)W);
  return t < 1 ? 1 : (t > W ? W : t);
}

// second threshold (Sec. 4.3); m1: mass of the retained prefix.
// returns 0 = nothing exact, 1 = every retained cluster, 2 = tau2 in [1, m1]
__device__ __forceinline__ int top_p_second_tau(float p2, bool p2_absolute, u64 W, u64 m1, u64 &tau2) {
  if (p2 >= 1.0f) return 1;
  if (p2 <= 0.0f) return 0;
  const u64 t = p2_absolute ? (u64)ceil((double)p2 * (double)W) : (u64)ceil((double)p2 * (double)m1);
  tau2 = t < 1 ? 1 : (t > m1 ? m1 : t);
  return 2;
}

}  // namespace dp
