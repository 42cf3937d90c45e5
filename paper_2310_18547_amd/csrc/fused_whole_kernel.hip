// Single-launch LoRA add-on for one-row segments without any hand-off between
// workgroups (gfx950).
//
// add_lora_fused_kernel splits the shrink of a segment over its S workgroups
// and pays for it with an exchange of partial sums through memory: about a
// microsecond at the end of a call in which nothing else is left to stream.
// Here every one of the S workgroups of a segment computes the WHOLE shrink
// v = x A_i itself and then expands its own column slice of B_i.  A_i is read S
// times, but only once from HBM: the launch places the S workgroups of a
// segment on ONE XCD, so the other S-1 reads are served by that XCD's L2, and
// each workgroup starts its walk over A_i at a different quarter so that the
// S workgroups fetch different parts first.  What it costs is address
// bandwidth of the compute unit's vector memory pipe (64 bytes per clock), of
// which the add-on leaves most idle anyway.
//
// Placement.  Workgroups go to the eight XCDs round-robin by linear id, and
// blockIdx.x is the fastest-varying part of that id, so a grid of (8, S, Q)
// puts workgroup (c, s, q) on XCD c; it serves segment q * 8 + c, slice s.
// Should a device deal workgroups differently the results are the same and only
// the L2 sharing is lost.
//
// No workspace, no generation count, no polling, nothing to time out: the workgroups of a
// launch never wait for each other, so the launch may be of any size.
#include <type_traits>

#include "device_common.h"
#include "exchange.h"
#include "launch.h"
#include "trace.h"

namespace sgmv {

// grid = (8, S, ceil(items / 8)) workgroups of 256 threads, items = segments (or rows, BY_ROW).
//   G = lane groups of the expand phase (group g multiplies weight rows g*R/G .. (g+1)*R/G-1)
//   U = 128-bit loads of A_i per lane and batch, all in flight together
// BY_ROW: the items of the grid are the n_tokens rows of the batch instead of its segments; a row's
// workgroups look its segment up (segment_of_row) and an XCD (blockIdx.x) takes a run of
// consecutive rows, so that small batches of longer segments with a small A_i run this kernel too.
template <class DT, int R, int G, int U, bool BY_ROW>
__global__ __launch_bounds__(256) void add_lora_whole_kernel(
    // the first sixteen dwords are preloaded into SGPRs at wave launch
    const int32_t* __restrict__ seg_starts, const uint16_t* const* __restrict__ A_ptrs,
    const uint16_t* const* __restrict__ B_ptrs, const uint16_t* __restrict__ x,
    uint16_t* __restrict__ y, int cslice, int h_in, int h_out, int n_segs, long long offA,
    long long offB, float scale, unsigned long long* header, int n_tokens) {
  constexpr int NT = 256, NW = 4;
  constexpr int LPR = R / 8;
  constexpr int CPW = NT / G;  // 8-column chunks per pass
  constexpr int JL = R / G;    // weight rows per lane in the expand phase
  constexpr int XL = kWholeMaxHin / (8 * NT);  // 128-bit x loads per lane
  static_assert(JL >= 1 && JL <= 16, "bad lane-group count");
  // two lane groups: neighbouring lanes, summed with a cross-lane move; more: whole waves per
  // group, summed through LDS (as in add_lora_fused_kernel, where the reasons are given)
  constexpr bool INTRA = G == 2;

  __shared__ __align__(16) uint16_t xs[kWholeMaxHin];
  __shared__ __align__(16) float red[NW][R];
  __shared__ __align__(16) float ex[(G > 2 ? (G - 1) : 1) * CPW * 8];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  SGMV_TRACE_DECL
  SGMV_TRACE_POINT(0);
  const int s = blockIdx.y, S = gridDim.y;
  int seg, lo, hi;
  if constexpr (BY_ROW) {
    const int row = blockIdx.x * gridDim.z + blockIdx.z;
    if (row >= n_tokens) return;
    seg = segment_of_row(seg_starts, n_segs, row, lane);
    if (seg >= n_segs) return;  // a row behind the last segment end
    lo = row;
    hi = row + 1;
  } else {
    seg = blockIdx.z * 8 + blockIdx.x;
    if (seg >= n_segs) return;
    lo = seg_starts[seg];
    hi = seg_starts[seg + 1];
  }
  const uint16_t* A = A_ptrs[seg];
  const uint16_t* B = B_ptrs[seg];
  if (lo >= hi || A == nullptr || B == nullptr) return;
  SGMV_TRACE_POINT(8);

  // A_i is walked in `iters` steps of NT 128-bit loads, U steps per batch; the launch checked
  // that U divides iters, so every step of every batch is a whole step inside A_i
  const int iters = h_in * LPR / NT;
  const int nbatch = iters / U;
  const int rot = (int)((long long)iters * s / S);  // where this workgroup starts its walk
  const int col_lo = min(h_out, s * cslice);
  const int ncols = max(0, min(h_out, col_lo + cslice) - col_lo);
  const int npass = (ncols + CPW * 8 - 1) / (CPW * 8);  // 0 when the column slice is empty
  const int cg = INTRA ? tid % G : tid / CPW;           // lane group
  const int cc = INTRA ? tid / G : tid - cg * CPW;      // chunk within pass

  const __amdgpu_buffer_rsrc_t rA = make_buffer(A + offA, (uint32_t)iters * (NT * 16u));
  const __amdgpu_buffer_rsrc_t rB = make_buffer(
      B + offB + col_lo, ncols > 0 ? (uint32_t)((long long)(R - 1) * h_out + ncols) * 2u : 0u);
  const uint32_t b_row0 = (uint32_t)(cg * JL) * (uint32_t)h_out * 2u;
  const uint32_t row_bytes_out = (uint32_t)h_out * 2u;
  // step i of the walk covers chunks walk(i) * NT + tid
  auto walk = [&](int i) {
    const int it = i + rot;
    return it >= iters ? it - iters : it;
  };
  const uint32_t a_lane = (uint32_t)tid * 16u;
  const uint16_t* xs_lane = xs + tid / LPR;  // step `it` multiplies by xs_lane[it * NT / LPR]

  for (int row = lo; row < hi; ++row) {
    if (row != lo) lds_barrier();  // xs, red and ex are free again
    // ---- issue everything: x, the first batch of A_i, the B slice, y
    const __amdgpu_buffer_rsrc_t rX = make_buffer(x + (long long)row * h_in, (uint32_t)h_in * 2u);
    const __amdgpu_buffer_rsrc_t rY = make_buffer(y + (long long)row * h_out + col_lo, (uint32_t)ncols * 2u);
    uint4 xr[XL];
#pragma unroll
    for (int i = 0; i < XL; ++i) xr[i] = buffer_load128(rX, (uint32_t)(i * NT + tid) * 16u);  // zeros beyond the row
    uint4 a[U];
#pragma unroll
    for (int u = 0; u < U; ++u) a[u] = buffer_load128_at(rA, a_lane, (uint32_t)walk(u) * (NT * 16u));
    __builtin_amdgcn_sched_barrier(0);  // keep x and A ahead of B and y in the memory pipe
    uint4 b[JL];
    uint4 yq;
    {
      const bool active = cc * 8 < ncols;
#pragma unroll
      for (int j = 0; j < JL; ++j)
        b[j] = buffer_load128(rB, active ? b_row0 + (uint32_t)j * row_bytes_out + (uint32_t)cc * 16u : kOutOfRange);
      yq = buffer_load128(rY, (cg == 0 && active) ? (uint32_t)cc * 16u : kOutOfRange);
    }
    __builtin_amdgcn_sched_barrier(0);
    SGMV_TRACE_POINT(1);

    // ---- shrink: the whole of v = x A_i
#pragma unroll
    for (int i = 0; i < XL; ++i) store128(&xs[(i * NT + tid) * 8], xr[i]);
    lds_barrier();  // xs filled
    SGMV_TRACE_POINT(2);
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    for (int batch = 0; batch < nbatch; ++batch) {
      if (batch != 0) {
#pragma unroll
        for (int u = 0; u < U; ++u)
          a[u] = buffer_load128_at(rA, a_lane, (uint32_t)walk(batch * U + u) * (NT * 16u));
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float af[8];
        unpack8<DT>(a[u], af);
        const float xv = decode1<DT>(xs_lane[walk(batch * U + u) * (NT / LPR)]);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaf(xv, af[e], acc[e]);
      }
    }
    {
      int e;
      const float d = reduce_lanes8<LPR>(acc, lane, e);
      if (lane < R) red[wave][(lane % LPR) * 8 + e] = d;
    }
    SGMV_TRACE_POINT(3);
    lds_barrier();  // red filled
    float vj[JL];
#pragma unroll
    for (int j = 0; j < JL; ++j) {
      const int c = cg * JL + j;
      vj[j] = ((red[0][c] + red[1][c]) + red[2][c]) + red[3][c];
    }
    SGMV_TRACE_POINT(5);

    // ---- expand of this workgroup's column slice
    for (int pass = 0; pass < npass; ++pass) {
      const int c = pass * CPW + cc;  // 8-column chunk within the slice
      const bool active = c * 8 < ncols;
      if (pass != 0) {
#pragma unroll
        for (int j = 0; j < JL; ++j)
          b[j] = buffer_load128(rB, active ? b_row0 + (uint32_t)j * row_bytes_out + (uint32_t)c * 16u : kOutOfRange);
        yq = buffer_load128(rY, (cg == 0 && active) ? (uint32_t)c * 16u : kOutOfRange);
      }
      float o[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = 0.f;
#pragma unroll
      for (int j = 0; j < JL; ++j) {
        float bf[8];
        unpack8<DT>(b[j], bf);
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = fmaf(vj[j], bf[e], o[e]);
      }
      if (INTRA) {
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] += neighbour_lane(o[e]);
      } else if (G > 1) {
        if (pass != 0) lds_barrier();  // ex free
        if (cg > 0) {
          float* dst = &ex[((cg - 1) * CPW + cc) * 8];
          *reinterpret_cast<float4*>(dst) = make_float4(o[0], o[1], o[2], o[3]);
          *reinterpret_cast<float4*>(dst + 4) = make_float4(o[4], o[5], o[6], o[7]);
        }
        lds_barrier();  // ex filled
        if (cg == 0) {
#pragma unroll
          for (int g = 1; g < G; ++g) {
            const float* srcp = &ex[((g - 1) * CPW + cc) * 8];
            const float4 p0 = *reinterpret_cast<const float4*>(srcp);
            const float4 p1 = *reinterpret_cast<const float4*>(srcp + 4);
            o[0] += p0.x; o[1] += p0.y; o[2] += p0.z; o[3] += p0.w;
            o[4] += p1.x; o[5] += p1.y; o[6] += p1.z; o[7] += p1.w;
          }
        }
      }
      if (cg == 0) {
        float yf[8];
        unpack8<DT>(yq, yf);
        uint4 out;
        out.x = pack2<DT>(yf[0] + scale * o[0], yf[1] + scale * o[1]);
        out.y = pack2<DT>(yf[2] + scale * o[2], yf[3] + scale * o[3]);
        out.z = pack2<DT>(yf[4] + scale * o[4], yf[5] + scale * o[5]);
        out.w = pack2<DT>(yf[6] + scale * o[6], yf[7] + scale * o[7]);
        buffer_store128(rY, active ? (uint32_t)c * 16u : kOutOfRange, out);
      }
    }
  }
  SGMV_TRACE_POINT(6);
#ifdef SGMV_TRACE
  if (header != nullptr) {
    SGMV_TRACE_FLUSH(tid == 0, 0, 3);
    SGMV_TRACE_FLUSH(tid == 0, 5, 6);
    SGMV_TRACE_FLUSH(tid == 0, 8, 8);
  }
#endif
}

template <class DT, int R, int G, int U>
static hipError_t launch_whole_t(const WholeArgs& a, hipStream_t st) {
  if (a.by_rows)
    hipLaunchKernelGGL((add_lora_whole_kernel<DT, R, G, U, true>),
                       dim3(8u, (unsigned)a.S, (unsigned)((a.n_tokens + 7) / 8)), dim3(256), 0, st, a.seg_starts,
                       (const uint16_t* const*)a.A_ptrs, (const uint16_t* const*)a.B_ptrs, (const uint16_t*)a.x,
                       (uint16_t*)a.y, a.cslice, a.h_in, a.h_out, a.n_segs, a.offA, a.offB, a.scale, a.header,
                       a.n_tokens);
  else
    hipLaunchKernelGGL((add_lora_whole_kernel<DT, R, G, U, false>),
                       dim3(8u, (unsigned)a.S, (unsigned)((a.n_segs + 7) / 8)), dim3(256), 0, st, a.seg_starts,
                       (const uint16_t* const*)a.A_ptrs, (const uint16_t* const*)a.B_ptrs, (const uint16_t*)a.x,
                       (uint16_t*)a.y, a.cslice, a.h_in, a.h_out, a.n_segs, a.offA, a.offB, a.scale, a.header,
                       a.n_tokens);
  return hipGetLastError();
}

template <class DT, int R, int G>
static hipError_t launch_whole_u(const WholeArgs& a, hipStream_t st) {
  // as many loads of A_i per lane in flight as divide its steps: all of it up to 32
  const int iters = a.h_in * (R / 8) / 256;
  if (iters % 32 == 0) return launch_whole_t<DT, R, G, 32>(a, st);
  if (iters % 16 == 0) return launch_whole_t<DT, R, G, 16>(a, st);
  if (iters % 8 == 0) return launch_whole_t<DT, R, G, 8>(a, st);
  if (iters % 4 == 0) return launch_whole_t<DT, R, G, 4>(a, st);
  if (iters % 2 == 0) return launch_whole_t<DT, R, G, 2>(a, st);
  return launch_whole_t<DT, R, G, 1>(a, st);
}

template <class DT, int R>
static hipError_t launch_whole_g(const WholeArgs& a, hipStream_t st) {
  switch (a.G) {
    case 1: if constexpr (R <= 16) return launch_whole_u<DT, R, 1>(a, st); break;
    case 2: if constexpr (R <= 32) return launch_whole_u<DT, R, 2>(a, st); break;
    case 4: return launch_whole_u<DT, R, 4>(a, st);
    case 8: return launch_whole_u<DT, R, 8>(a, st);
  }
  return hipErrorInvalidValue;
}

template <class DT>
static hipError_t launch_whole_r(const WholeArgs& a, hipStream_t st) {
  switch (a.r) {
    case 8: return launch_whole_g<DT, 8>(a, st);
    case 16: return launch_whole_g<DT, 16>(a, st);
    case 32: return launch_whole_g<DT, 32>(a, st);
    case 64: return launch_whole_g<DT, 64>(a, st);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_add_lora_whole(const WholeArgs& a, hipStream_t st) {
  return a.bf16 ? launch_whole_r<BF16>(a, st) : launch_whole_r<F16>(a, st);
}

}  // namespace sgmv
