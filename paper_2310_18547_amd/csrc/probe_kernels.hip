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
//           reference for scaling FETCH_SIZE / WRITE_SIZE.
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
    default:
      return SGMV_ERR_UNSUPPORTED;
  }
  return hipGetLastError() == hipSuccess ? SGMV_OK : SGMV_ERR_LAUNCH;
}
