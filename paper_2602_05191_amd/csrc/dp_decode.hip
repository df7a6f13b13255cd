// Stage 3 as a kernel of its own: the queue of dp_decode_body.hpp over the plan that an earlier launch (the
// selection kernel, or the planner of caller-given sets) left in the workspace.
#include <hip/hip_ext.h>

#include "dp_decode_body.hpp"

namespace dp {
namespace {

constexpr int kDecThreads = 256;

template <bool kGathered>
__global__ __launch_bounds__(kDecThreads) void decode_kernel(const int32_t *pending, DecodeArgs a) {
  DP_DECODE_LDS(kDecThreads);
  // (a leading scalar parameter: it is in a register when the wave starts, so a launch that finds nothing to do
  // issues this load first and fetches no other argument)
  if (pending && *pending == 0) return;  // every head was finished by the selection kernel
  decode_queue<kDecThreads, kGathered, false>(a, DP_DECODE_LDS_ARGS);
}

}  // namespace

hipError_t launch_decode(const CacheView &c, const int32_t *n_exact, const int32_t *n_retained, const Plan &plan,
                         float *partials, int splits, const AttnOut &attn, hipStream_t s, hipEvent_t start,
                         hipEvent_t stop, const void *k_gather, const void *v_gather, int rows_cap) {
  const int nh = c.batch * c.n_q_heads;
  if (nh == 0) return hipSuccess;
  DecodeArgs a = decode_args_of(c, n_exact, n_retained, plan, partials, splits, attn);
  a.k_gather = k_gather;
  a.v_gather = v_gather;
  a.rows_cap = rows_cap;
  // one launch per slab of kMaxQueueHeads heads, each with its own item counter
  for (int h0 = 0, slab = 0; h0 < nh; h0 += kMaxQueueHeads, ++slab) {
    a.head0 = h0;
    a.n_heads = nh - h0 < kMaxQueueHeads ? nh - h0 : kMaxQueueHeads;
    a.queue_next = plan.queue_next + slab;
    a.pending = plan.pending ? plan.pending + slab : nullptr;
    const long max_items = (long)a.n_heads * splits;
    const int grid = (int)(max_items < kDecodeGrid ? max_items : kDecodeGrid);
    // measurement: the events bracket the first slab's begin and the last slab's end
    hipEvent_t ev0 = (h0 == 0) ? start : nullptr, ev1 = (h0 + kMaxQueueHeads >= nh) ? stop : nullptr;
    if (k_gather)
      hipLaunchKernelGGL(decode_kernel<true>, dim3(grid), dim3(kDecThreads), 0, s, a.pending, a);
    else if (ev0 || ev1)
      hipExtLaunchKernelGGL(decode_kernel<false>, dim3(grid), dim3(kDecThreads), 0, s, ev0, ev1, 0, a.pending, a);
    else
      hipLaunchKernelGGL(decode_kernel<false>, dim3(grid), dim3(kDecThreads), 0, s, a.pending, a);
  }
  return hipGetLastError();
}

}  // namespace dp
