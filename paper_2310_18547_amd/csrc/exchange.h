// Cross-workgroup hand-off helpers of the single-launch kernels (gfx950).
//
// Partial sums travel between the workgroups of one launch as 64-bit words
// {fp32 value (high half), generation tag (low half)} written and read with
// agent-scope accesses (the L2s of the eight XCDs are not coherent with each
// other).  The tag is the launch's generation number, derived from an epoch
// kept in the workspace: every workgroup of a launch adds to the epoch on exit
// so that the launch advances it by exactly kEpochStep in total; while a launch
// runs, epoch / kEpochStep is therefore the same for all of its workgroups.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "launch.h"

namespace sgmv {

// Workgroup barrier that orders LDS traffic only: outstanding global loads stay
// outstanding.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ uint32_t generation_tag(unsigned long long epoch) {
  return (uint32_t)((epoch / kEpochStep) % 0xFFFFFFFFull) + 1u;  // never 0
}

// Each workgroup adds to the epoch exactly once, on its way out; the first
// workgroup adds the remainder so that the launch's total is kEpochStep.  The
// epoch is the sum of kEpochCounters words and a workgroup adds to the word
// its id selects, which spreads the atomics over many addresses.
__device__ __forceinline__ void leave_launch(unsigned long long* epoch, int n_workgroups) {
  const unsigned id = (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
  const unsigned long long inc =
      id == 0 ? (unsigned long long)kEpochStep - (n_workgroups - 1) : 1ull;
  __hip_atomic_fetch_add(epoch + (id % kEpochCounters), inc, __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
}

// Read the epoch with one wave: lane l reads counter l, the lanes are summed.
// The counters only grow, and this workgroup has not added its share yet, so
// whatever mixture of old and new counter values the lanes see, the sum lies
// in the running launch's window.
__device__ __forceinline__ unsigned long long read_epoch(const unsigned long long* epoch, int lane) {
  static_assert(kEpochCounters == 64, "one counter per lane");
  unsigned long long v = __hip_atomic_load(epoch + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) {
    const unsigned lo = __shfl_xor((unsigned)v, m, 64);
    const unsigned hi = __shfl_xor((unsigned)(v >> 32), m, 64);
    v += ((unsigned long long)hi << 32) | lo;
  }
  return v;
}

// Consumer side of the hand-off for one element: poll the S words at src, src + stride, ...
// until all carry `tag`, and return the sum of their values in ascending slice order.  Gives
// up after spin_limit incomplete polls (sets timed_out; the sum is then meaningless).
//
// One poll is a round trip to the memory side (about half a microsecond), so fresh data is
// seen up to one round trip late.  Keeping several polls in flight, a fraction of a round
// trip apart, was tried: hipcc's wait-count insertion loses track of the ring in the loop
// and waits for every outstanding poll before each examination, which made the call 0.5 us
// slower; the plain loop stays.
__device__ __forceinline__ float collect_slices(const unsigned long long* src, long long stride, int S,
                                                uint32_t tag, int spin_limit, bool& timed_out) {
  float sum = 0.f;
  for (int s0 = 0; s0 < S; s0 += 8) {
    unsigned long long wv[8];
    int polls = 0;
    bool ready;
    do {
#pragma unroll
      for (int i = 0; i < 8; ++i)
        wv[i] = __hip_atomic_load(src + (long long)min(s0 + i, S - 1) * stride, __ATOMIC_RELAXED,
                                  __HIP_MEMORY_SCOPE_AGENT);
      ready = true;
#pragma unroll
      for (int i = 0; i < 8; ++i) ready = ready && ((uint32_t)wv[i] == tag);
      if (!ready && ++polls > spin_limit) {
        timed_out = true;
        break;
      }
    } while (!ready);
#pragma unroll
    for (int i = 0; i < 8; ++i) sum += (s0 + i < S) ? __uint_as_float((uint32_t)(wv[i] >> 32)) : 0.f;
  }
  return sum;
}

}  // namespace sgmv
