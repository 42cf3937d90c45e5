// Cross-workgroup hand-off helpers of the single-launch kernels (gfx950).
//
// Partial sums travel between the workgroups of one launch as 64-bit words
// {fp32 value (high half), generation tag (low half)} written and read with
// agent-scope accesses (the L2s of the eight XCDs are not coherent with each
// other).  The tag is the workspace's generation: the number of single-launch
// kernels that have run on it (never zero).  A consumer polls a word until its
// tag is the running launch's generation, so there is no separate flag and
// nothing to reset: what an earlier launch left behind carries an older tag.
//
// The generation lives at the start of the workspace in kGenerationCopies
// identical copies.  Workgroup i (linear id) of a launch of n workgroups reads
// copy i when it starts and writes generation + 1 to the copies i, i + n,
// i + 2n, ... when it leaves.  Only workgroup i of the running launch writes
// copy i, and only on its way out, so every workgroup reads the value the
// previous launch left; and when a launch has ended all copies agree again,
// whatever its size.  (The first design summed 64 counters to which the
// workgroups added on exit: every workgroup's read then went to the same 512
// bytes, which with 256 workgroups took 2.4 us at the median and held up the
// hand-off by 0.45 us.)
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "device_common.h"
#include "launch.h"

namespace sgmv {

__device__ __forceinline__ unsigned workgroup_linear_id() {
  return (blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
}
__device__ __forceinline__ uint32_t* generation_copies(unsigned long long* header) {
  return reinterpret_cast<uint32_t*>(header);
}
__device__ __forceinline__ uint32_t* error_word(unsigned long long* header) {
  return reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(header) + kWorkspaceErrorOffset);
}
__device__ __forceinline__ void raise_timeout(unsigned long long* header) {
  __hip_atomic_store(error_word(header), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The running launch's generation tag (wave-uniform); call with a whole wave.
__device__ __forceinline__ uint32_t launch_tag(unsigned long long* header) {
  const uint32_t g = __hip_atomic_load(generation_copies(header) + workgroup_linear_id(), __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
  return __builtin_amdgcn_readfirstlane(g);
}

// A workgroup's last act, by one whole wave: advance its copies of the generation.
__device__ __forceinline__ void leave_launch(unsigned long long* header, int n_workgroups, uint32_t tag,
                                             int lane) {
  const uint32_t next = tag + 1u == 0u ? 1u : tag + 1u;
  uint32_t* copies = generation_copies(header);
  for (int k = (int)workgroup_linear_id() + lane * n_workgroups; k < kGenerationCopies; k += 64 * n_workgroups)
    __hip_atomic_store(copies + k, next, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// The same for a workgroup that has nothing to do and never asked for the tag.
__device__ __forceinline__ void leave_launch_idle(unsigned long long* header, int n_workgroups, int lane) {
  leave_launch(header, n_workgroups, launch_tag(header), lane);
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
      if (!ready && ++polls >= spin_limit) {
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
