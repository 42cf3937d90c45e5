// In-kernel timeline probe of the single-launch kernels (tuning builds only).
//
// Built with -DSGMV_TRACE (python -m paper_2310_18547_amd.build --trace -> libsgmv_trace.so)
// every workgroup records the constant-rate device clock (100 MHz) at up to ten marked
// points in registers and writes them out when its waves leave:
//     buffer[workgroup * 10 + point]
// where `buffer` is the device address found in the 64-bit word eight bytes behind the error
// word of the workspace header (zero = tracing off; sgmv_workspace_init clears it).  Without the
// macro SGMV_TRACE the three hooks expand to nothing and the library carries no trace code.
//
// Points of add_lora_fused_kernel / add_lora_tile_kernel:
//   0 workgroup started            8 segment bounds and weight pointers known
//   1 all up-front loads issued    2 x (and, tile kernel, the A slice) staged in LDS
//   3 shrink of the slice done     4 partial sums published (exchange wave)
//   5 all slices collected         6 y stored (stream waves done)
//   7 exchange wave leaves          9 address arithmetic done, first load about to issue
//                                     (tile kernel only)
#pragma once
#include <hip/hip_runtime.h>

#include "launch.h"

#ifdef SGMV_TRACE
#define SGMV_TRACE_DECL \
  unsigned long long trace_ts[10] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#define SGMV_TRACE_POINT(point)          \
  do {                                   \
    trace_ts[point] = wall_clock64();    \
  } while (0)
#define SGMV_TRACE_FLUSH(cond, first, last)                                                       \
  do {                                                                                            \
    unsigned long long* trace_buf = reinterpret_cast<unsigned long long*>(                        \
        __hip_atomic_load(reinterpret_cast<unsigned long long*>(                                  \
                              reinterpret_cast<char*>(header) + sgmv::kWorkspaceTraceOffset),     \
                          __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));                           \
    if (trace_buf != nullptr && (cond)) {                                                         \
      const size_t trace_wg =                                                                     \
          ((size_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;                 \
      for (int tp = (first); tp <= (last); ++tp) trace_buf[trace_wg * 10 + tp] = trace_ts[tp];    \
    }                                                                                             \
  } while (0)
#else
#define SGMV_TRACE_DECL
#define SGMV_TRACE_POINT(point)
#define SGMV_TRACE_FLUSH(cond, first, last)
#endif
