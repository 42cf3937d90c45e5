// Measurement aids of libsgmv: plain kernels of known traffic (gfx950).
//
// The SGMV kernels are judged against what this GPU delivers to a kernel that does nothing
// but move the same bytes, and rocprofv3's HBM byte counters are scaled by what they read
// for a copy of known size.  These are those kernels, behind one C entry point so that the
// benchmark and the profiles use the library that is being measured:
//   kind 0  empty kernel, one workgroup of 320 threads per compute-unit-sized share
//           (the launch shape of the single-launch add-on): the cost of a launch;
//   kind 1  streaming read of `bytes` from `src`: workgroups of 256 threads, each reading
//           contiguous 64 KiB chunks with sixteen 128-bit loads per lane in flight (the
//           access pattern of a workgroup's weight slices); the attainable read bandwidth
//           for a launch that moves `bytes`;
//   kind 2  copy of `bytes` from `src` to `dst` (reads `bytes`, writes `bytes`): the
//           reference for scaling FETCH_SIZE / WRITE_SIZE;
//   kind 3  round trips of a 64-bit word between two workgroups with the accesses of the
//           single-launch kernels' hand-off: what one hop of that hand-off costs at least.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sgmv.h"
#include "device_common.h"

namespace sgmv {

constexpr int kProbeLoads = 16;                      // 128-bit loads per lane in flight
constexpr size_t kProbeChunk = 256 * kProbeLoads * 16;  // bytes per workgroup and step (64 KiB)

__global__ __launch_bounds__(320) void probe_empty_kernel() {}

__global__ __launch_bounds__(256) void probe_read_kernel(const uint4* __restrict__ src, size_t n_chunks,
                                                         size_t bytes, uint32_t* sink) {
  uint32_t acc = 0;
  for (size_t chunk = blockIdx.x; chunk < n_chunks; chunk += gridDim.x) {
    const size_t first = chunk * kProbeChunk;
    const size_t left = bytes - first;
    const __amdgpu_buffer_rsrc_t rs = make_buffer(
        reinterpret_cast<const char*>(src) + first, (uint32_t)(left < kProbeChunk ? left : kProbeChunk));
    uint4 v[kProbeLoads];
#pragma unroll
    for (int u = 0; u < kProbeLoads; ++u) v[u] = buffer_load128(rs, (uint32_t)(u * 256 + threadIdx.x) * 16u);
#pragma unroll
    for (int u = 0; u < kProbeLoads; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x9E3779B9u && sink != nullptr) sink[0] = acc;  // keeps the loads; practically never taken
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                         size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = src[i];
}

// Round trips of one 64-bit word between two workgroups of a launch, written and polled with
// the agent-scope accesses of the single-launch kernels' hand-off: workgroup 0 and workgroup
// `partner` of a grid of 64 answer each other kProbeRounds times; the others leave at once.
// Workgroups go to the eight XCDs round-robin, so partner 8 shares workgroup 0's XCD and
// partner 1 sits on the next one.  out[0] = ticks of the 100 MHz device clock for all rounds,
// out[1] = 1 if a wait was given up (every wait is bounded).
constexpr int kProbeRounds = 200;
__global__ __launch_bounds__(64) void probe_handoff_kernel(unsigned long long* words, int partner,
                                                           unsigned long long* out) {
  const int id = blockIdx.x;
  if ((id != 0 && id != partner) || threadIdx.x != 0) return;
  unsigned long long* mine = words + (id == 0 ? 0 : 32);  // separate cache lines
  unsigned long long* theirs = words + (id == 0 ? 32 : 0);
  // the words may hold an earlier call's count: start above whatever is there
  const unsigned long long base = __hip_atomic_load(words + 16, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const unsigned long long t0 = wall_clock64();
  for (int r = 1; r <= kProbeRounds; ++r) {
    const unsigned long long want = base + (unsigned long long)r;
    if (id == 0) __hip_atomic_store(mine, want, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int polls = 0;
    while (__hip_atomic_load(theirs, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != want) {
      if (++polls > (1 << 16)) {
        out[1] = 1;
        return;
      }
    }
    if (id != 0) __hip_atomic_store(mine, want, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  if (id == 0) {
    out[0] = wall_clock64() - t0;
    __hip_atomic_store(words + 16, base + kProbeRounds, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

}  // namespace sgmv

extern "C" int sgmv_probe(int kind, const void* src, void* dst, size_t bytes, void* stream) {
  using namespace sgmv;
  hipStream_t st = static_cast<hipStream_t>(stream);
  int dev = 0, cu = 256;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu <= 0)
    return SGMV_ERR_LAUNCH;
  switch (kind) {
    case 0:
      hipLaunchKernelGGL(probe_empty_kernel, dim3((unsigned)cu), dim3(320), 0, st);
      break;
    case 1: {
      if (src == nullptr) return SGMV_ERR_NULL;
      if (bytes == 0 || bytes % 16 != 0 || (reinterpret_cast<uintptr_t>(src) & 15) != 0) return SGMV_ERR_ALIGN;
      const size_t n_chunks = (bytes + kProbeChunk - 1) / kProbeChunk;
      const size_t most = (size_t)cu * 8;
      hipLaunchKernelGGL(probe_read_kernel, dim3((unsigned)(n_chunks < most ? n_chunks : most)), dim3(256), 0,
                         st, static_cast<const uint4*>(src), n_chunks, bytes, static_cast<uint32_t*>(dst));
      break;
    }
    case 2: {
      if (src == nullptr || dst == nullptr) return SGMV_ERR_NULL;
      if (bytes == 0 || bytes % 16 != 0 || (reinterpret_cast<uintptr_t>(src) & 15) != 0 ||
          (reinterpret_cast<uintptr_t>(dst) & 15) != 0)
        return SGMV_ERR_ALIGN;
      const size_t n = bytes / 16;
      const size_t blocks = (n + 255) / 256;
      const size_t most = (size_t)cu * 8;
      hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)(blocks < most ? blocks : most)), dim3(256), 0, st,
                         static_cast<const uint4*>(src), static_cast<uint4*>(dst), n);
      break;
    }
    case 3: {
      if (src == nullptr || dst == nullptr) return SGMV_ERR_NULL;
      if ((reinterpret_cast<uintptr_t>(src) & 255) != 0 || (reinterpret_cast<uintptr_t>(dst) & 15) != 0)
        return SGMV_ERR_ALIGN;
      if (bytes < 1 || bytes > 63) return SGMV_ERR_SHAPE;
      hipLaunchKernelGGL(probe_handoff_kernel, dim3(64), dim3(64), 0, st,
                         static_cast<unsigned long long*>(const_cast<void*>(src)), (int)bytes,
                         static_cast<unsigned long long*>(dst));
      break;
    }
    default:
      return SGMV_ERR_UNSUPPORTED;
  }
  return hipGetLastError() == hipSuccess ? SGMV_OK : SGMV_ERR_LAUNCH;
}
