// Stand-alone SGMV shrink for one-row segments in a single launch without Split-K, gfx950.
//
// v[row] += x[row] A_i (section "Segmented Gather Matrix-Vector Multiplication", the shrink
// launch).  The paper splits the shrink along h_in for parallelism; a batch of a few hundred
// one-row segments has that parallelism in its segments, so here one workgroup computes the
// whole product of its segment (the shrink phase of fused_whole_kernel.hip: all of A_i in flight at
// once, up to 32 128-bit loads per lane) and adds it to the caller's v itself: no partial sums,
// no second launch that adds them up, no workspace.
#include "device_common.h"
#include "launch.h"

namespace sgmv {

// grid = n_segs workgroups of 256 threads.  U = 128-bit loads of A_i per lane and batch, all in
// flight together; the launch picks the largest U of 32 .. 1 with h_in * R / 8 a multiple of 256 * U.
// BY_ROW: grid = the rows of the batch rounded up to a multiple of eight; a workgroup serves one row
// and looks the row's segment up (n_segs of them), blockIdx.x % 8, the XCD it lands on, taking a run
// of consecutive rows, which then find their segment's A_i in one L2.
template <class DT, int R, int U, bool BY_ROW>
__global__ __launch_bounds__(256) void shrink_whole_kernel(
    const int32_t* __restrict__ seg_starts, const uint16_t* const* __restrict__ A_ptrs,
    const uint16_t* __restrict__ x, float* __restrict__ v, int h_in, long long offA, int n_tokens, int n_segs) {
  constexpr int NT = 256, NW = 4;
  constexpr int LPR = R / 8;
  constexpr int XL = kWholeMaxHin / (8 * NT);  // 128-bit x loads per lane
  __shared__ __align__(16) uint16_t xs[kWholeMaxHin];
  __shared__ __align__(16) float red[NW][R];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int seg = blockIdx.x, lo, hi;
  if constexpr (BY_ROW) {
    const int row = ((int)blockIdx.x & 7) * ((int)gridDim.x >> 3) + ((int)blockIdx.x >> 3);
    if (row >= n_tokens) return;
    seg = segment_of_row(seg_starts, n_segs, row, lane);
    if (seg >= n_segs) return;  // a row behind the last segment end
    lo = row;
    hi = row + 1;
  } else {
    lo = seg_starts[seg];
    hi = seg_starts[seg + 1];
  }
  const uint16_t* A = A_ptrs[seg];
  if (lo >= hi || A == nullptr) return;

  const int iters = h_in * LPR / NT;  // steps of NT 128-bit loads over A_i
  const int nbatch = iters / U;
  const __amdgpu_buffer_rsrc_t rA = make_buffer(A + offA, (uint32_t)iters * (NT * 16u));
  const uint32_t a_lane = (uint32_t)tid * 16u;
  const uint16_t* xs_lane = xs + tid / LPR;  // step `it` multiplies by xs_lane[it * NT / LPR]

  for (int row = lo; row < hi; ++row) {
    if (row != lo) lds_barrier();  // xs and red are free again
    const __amdgpu_buffer_rsrc_t rX = make_buffer(x + (long long)row * h_in, (uint32_t)h_in * 2u);
    uint4 xr[XL];
#pragma unroll
    for (int i = 0; i < XL; ++i) xr[i] = buffer_load128(rX, (uint32_t)(i * NT + tid) * 16u);  // zeros beyond the row
    uint4 a[U];
#pragma unroll
    for (int u = 0; u < U; ++u) a[u] = buffer_load128_at(rA, a_lane, (uint32_t)u * (NT * 16u));
    const float before = tid < R ? v[(long long)row * R + tid] : 0.f;
#pragma unroll
    for (int i = 0; i < XL; ++i) store128(&xs[(i * NT + tid) * 8], xr[i]);
    lds_barrier();  // xs filled

    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    for (int batch = 0; batch < nbatch; ++batch) {
      if (batch != 0) {
#pragma unroll
        for (int u = 0; u < U; ++u) a[u] = buffer_load128_at(rA, a_lane, (uint32_t)(batch * U + u) * (NT * 16u));
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float af[8];
        unpack8<DT>(a[u], af);
        const float xv = decode1<DT>(xs_lane[(batch * U + u) * (NT / LPR)]);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaf(xv, af[e], acc[e]);
      }
    }
    {
      int e;
      const float d = reduce_lanes8<LPR>(acc, lane, e);
      if (lane < R) red[wave][(lane % LPR) * 8 + e] = d;
    }
    lds_barrier();  // red filled
    if (tid < R) v[(long long)row * R + tid] = before + (((red[0][tid] + red[1][tid]) + red[2][tid]) + red[3][tid]);
  }
}

template <class DT, int R, int U>
static hipError_t launch_shrink_whole_t(const ShrinkArgs& a, hipStream_t st, float* v) {
  if (a.by_rows)
    hipLaunchKernelGGL((shrink_whole_kernel<DT, R, U, true>), dim3((unsigned)((a.n_tokens + 7) / 8 * 8)), dim3(256), 0, st,
                       a.seg_starts, (const uint16_t* const*)a.A_ptrs, (const uint16_t*)a.x, v, a.h_in, a.layer_off,
                       a.n_tokens, a.n_segs);
  else
    hipLaunchKernelGGL((shrink_whole_kernel<DT, R, U, false>), dim3((unsigned)a.n_segs), dim3(256), 0, st, a.seg_starts,
                       (const uint16_t* const*)a.A_ptrs, (const uint16_t*)a.x, v, a.h_in, a.layer_off, a.n_tokens,
                       a.n_segs);
  return hipGetLastError();
}

template <class DT, int R>
static hipError_t launch_shrink_whole_u(const ShrinkArgs& a, hipStream_t st, float* v) {
  // as many loads of A_i per lane in flight as divide its steps: all of it up to 32
  const int iters = a.h_in * (R / 8) / 256;
  if (iters % 32 == 0) return launch_shrink_whole_t<DT, R, 32>(a, st, v);
  if (iters % 16 == 0) return launch_shrink_whole_t<DT, R, 16>(a, st, v);
  if (iters % 8 == 0) return launch_shrink_whole_t<DT, R, 8>(a, st, v);
  if (iters % 4 == 0) return launch_shrink_whole_t<DT, R, 4>(a, st, v);
  if (iters % 2 == 0) return launch_shrink_whole_t<DT, R, 2>(a, st, v);
  return launch_shrink_whole_t<DT, R, 1>(a, st, v);
}

template <class DT>
static hipError_t launch_shrink_whole_r(const ShrinkArgs& a, hipStream_t st, float* v) {
  switch (a.r) {
    case 8: return launch_shrink_whole_u<DT, 8>(a, st, v);
    case 16: return launch_shrink_whole_u<DT, 16>(a, st, v);
    case 32: return launch_shrink_whole_u<DT, 32>(a, st, v);
    case 64: return launch_shrink_whole_u<DT, 64>(a, st, v);
  }
  return hipErrorInvalidValue;
}

bool shrink_whole_fits(const ShrinkArgs& a) {
  return a.h_in <= kWholeMaxHin && (long long)a.h_in * (a.r / 8) % 256 == 0 && a.n_segs > 0;
}

hipError_t launch_shrink_whole(const ShrinkArgs& a, float* v, hipStream_t st) {
  if (!shrink_whole_fits(a) || v == nullptr) return hipErrorInvalidValue;
  return a.bf16 ? launch_shrink_whole_r<BF16>(a, st, v) : launch_shrink_whole_r<F16>(a, st, v);
}

}  // namespace sgmv
