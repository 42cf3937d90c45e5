// Stand-alone SGMV shrink for one-row segments in a single launch, gfx950.
//
// v[row] += x[row] A_i (section "Segmented Gather Matrix-Vector Multiplication", the shrink
// launch with Split-K).  With the launch-per-step kernels the Split-K partial sums cost a
// second launch that adds them up; here the S workgroups of a segment hand their partial
// sums to the first of them inside the launch, as in the single-launch add-on
// (fused_kernel.hip, whose shrink phase this is): 64-bit {value, generation tag} words,
// agent-scope accesses, a fifth wave that polls so that it never queues behind streaming
// loads, a bounded wait.  Only the workgroup of slice 0 collects; the others leave as soon
// as they have published.  The sums are added in ascending slice order and then to the
// caller's v, exactly as the two-launch path does.
#include "device_common.h"
#include "exchange.h"
#include "launch.h"

namespace sgmv {

// grid (fused_grid_x, S, rows of segments), 320 threads: four stream waves, one exchange wave.
//   exch   [S][n_tokens][R] 64-bit words {fp32 value (high), tag (low)}
// BY_ROW: the grid's items are the n_tokens rows of the batch, not its segments; a row's
// workgroups look the row's segment up in seg_starts, so segments may have any length, and an
// XCD (blockIdx.x) takes a run of consecutive rows (as in the add-on kernel, fused_kernel.hip).
template <class DT, int R, bool BY_ROW>
__global__ __launch_bounds__(320) void shrink_handoff_kernel(
    const int32_t* __restrict__ seg_starts, const uint16_t* const* __restrict__ A_ptrs,
    const uint16_t* __restrict__ x, float* __restrict__ v, int kslice, int h_in, int n_tokens, int S,
    long long offA, unsigned long long* exch, unsigned long long* header, int spin_limit, int n_segs) {
  constexpr int NT = 256, NW = 4, U = 8;  // stream threads / waves, A loads per lane and batch
  constexpr int LPR = R / 8;
  static_assert(kMaxKSlice / 8 == NT, "one 128-bit x chunk per lane");
  __shared__ __align__(16) uint16_t xs[kMaxKSlice];
  __shared__ __align__(16) float red[NW * 4][R];  // per wave and row of sixteen lanes

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_workgroups = (int)(gridDim.x * gridDim.y * gridDim.z);
  // blockIdx.x is the fastest-varying part of the linear id by which workgroups are dealt to
  // the XCDs, so the S workgroups of a segment share an XCD
  const int item = BY_ROW ? blockIdx.x * gridDim.z + blockIdx.z : blockIdx.z * gridDim.x + blockIdx.x;
  const int s = blockIdx.y;
  if (item >= (BY_ROW ? n_tokens : n_segs)) {  // the grid is padded to whole rows of items
    if (wave == 0) leave_launch_idle(header, n_workgroups, lane);
    return;
  }
  int lo, hi;
  const uint16_t* A;
  if constexpr (BY_ROW) {
    const int found = segment_of_row(seg_starts, n_segs, item, lane);
    lo = item;
    hi = found < n_segs ? item + 1 : item;  // a row behind the last segment end: nothing to do
    A = found < n_segs ? A_ptrs[found] : nullptr;
  } else {
    lo = seg_starts[item];
    hi = seg_starts[item + 1];
    A = A_ptrs[item];
  }
  if (lo >= hi || A == nullptr) {  // same decision in all S workgroups
    if (wave == 0) leave_launch_idle(header, n_workgroups, lane);
    return;
  }
  const int k0 = s * kslice;
  const int klen = max(0, min(h_in, k0 + kslice) - k0);
  const int nchunks = klen * LPR;  // 128-bit chunks in this workgroup's slice of A_i
  const long long stride = (long long)n_tokens * R;

  // One row per segment is what the caller promised (the length hint); a longer segment is still
  // covered, row after row, each with its own hand-off.
  if (wave == NW) {
    // ============================================================ exchange wave
    const uint32_t tag = launch_tag(header);
    bool timed_out = false;
    for (int row = lo; row < hi; ++row) {
      if (row != lo) lds_barrier();  // (a) xs / red free
      lds_barrier();                 // (b) xs filled
      lds_barrier();                 // (c) red filled
      if (lane < R) {
        float sum = red[0][lane];
#pragma unroll
        for (int w = 1; w < NW * 4; ++w) sum += red[w][lane];
        const unsigned long long word = ((unsigned long long)__float_as_uint(sum) << 32) | tag;
        __hip_atomic_store(exch + (long long)s * stride + (long long)row * R + lane, word, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
      }
      if (s == 0 && lane < R) {
        const float before = v[(long long)row * R + lane];  // in flight with the first poll
        bool gave_up = false;
        const float sum = collect_slices(exch + (long long)row * R + lane, stride, S, tag, spin_limit, gave_up);
        if (!gave_up) v[(long long)row * R + lane] = before + sum;  // an incomplete sum is never stored
        timed_out = timed_out || gave_up;
      }
    }
    if (__any(timed_out)) raise_timeout(header);
    leave_launch(header, n_workgroups, tag, lane);
    return;
  }

  // ================================================================ stream waves
  const int cpr = klen >> 3;  // 128-bit chunks in the x row slice
  const __amdgpu_buffer_rsrc_t rA = make_buffer(A + offA + (long long)k0 * R, (uint32_t)nchunks * 16u);
  for (int row = lo; row < hi; ++row) {
    const __amdgpu_buffer_rsrc_t rX = make_buffer(x + (long long)row * h_in + k0, (uint32_t)klen * 2u);
    const uint4 xr = buffer_load128(rX, tid < cpr ? (uint32_t)tid * 16u : kOutOfRange);
    uint4 a[U];
#pragma unroll
    for (int u = 0; u < U; ++u) a[u] = buffer_load128(rA, (uint32_t)(u * NT + tid) * 16u);
    if (row != lo) lds_barrier();  // (a) xs / red free
    // chunks that do not exist arrive as zeros, so xs is always fully defined
    store128(&xs[tid * 8], xr);
    lds_barrier();  // (b) xs filled

    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    for (int base = 0; base < nchunks; base += NT * U) {
      if (base != 0) {
#pragma unroll
        for (int u = 0; u < U; ++u) a[u] = buffer_load128(rA, (uint32_t)(base + u * NT + tid) * 16u);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int q = base + u * NT + tid;
        const int kk = (q / LPR) & (kMaxKSlice - 1);
        float af[8];
        unpack8<DT>(a[u], af);
        const float xraw = decode1<DT>(xs[kk]);
        const float xv = (q < nchunks) ? xraw : 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaf(xv, af[e], acc[e]);
      }
    }
    // Lane l holds partial sums of the columns (l % LPR) * 8 .. + 7: summed over each row of
    // sixteen lanes in the vector ALU, then over the sixteen rows of the workgroup by the
    // exchange wave, in a fixed order.
    float d[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) d[e] = row_sum_same_group<LPR>(acc[e]);
    if ((lane & 15) < LPR) {
      float* dst = &red[wave * 4 + (lane >> 4)][(lane & 15) * 8];
      *reinterpret_cast<float4*>(dst) = make_float4(d[0], d[1], d[2], d[3]);
      *reinterpret_cast<float4*>(dst + 4) = make_float4(d[4], d[5], d[6], d[7]);
    }
    lds_barrier();  // (c) red filled
  }
}

template <class DT, int R, bool BY_ROW>
static hipError_t launch_shrink_handoff_b(const FusedArgs& a, float* v, hipStream_t st) {
  const int items = BY_ROW ? a.n_tokens : a.n_segs;
  const int gx = fused_grid_x(items);
  hipLaunchKernelGGL((shrink_handoff_kernel<DT, R, BY_ROW>), dim3((unsigned)gx, (unsigned)a.S, (unsigned)((items + gx - 1) / gx)),
                     dim3(320), 0, st, a.seg_starts, (const uint16_t* const*)a.A_ptrs, (const uint16_t*)a.x, v,
                     a.kslice, a.h_in, a.n_tokens, a.S, a.offA, a.exch, a.header, a.spin_limit, a.n_segs);
  return hipGetLastError();
}

template <class DT, int R>
static hipError_t launch_shrink_handoff_t(const FusedArgs& a, float* v, hipStream_t st) {
  return a.by_rows ? launch_shrink_handoff_b<DT, R, true>(a, v, st) : launch_shrink_handoff_b<DT, R, false>(a, v, st);
}

template <class DT>
static hipError_t launch_shrink_handoff_r(const FusedArgs& a, float* v, hipStream_t st) {
  switch (a.r) {
    case 8: return launch_shrink_handoff_t<DT, 8>(a, v, st);
    case 16: return launch_shrink_handoff_t<DT, 16>(a, v, st);
    case 32: return launch_shrink_handoff_t<DT, 32>(a, v, st);
    case 64: return launch_shrink_handoff_t<DT, 64>(a, v, st);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_shrink_handoff(const FusedArgs& a, float* v, hipStream_t st) {
  return a.bf16 ? launch_shrink_handoff_r<BF16>(a, v, st) : launch_shrink_handoff_r<F16>(a, v, st);
}

}  // namespace sgmv
