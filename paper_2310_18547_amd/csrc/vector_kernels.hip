// Bandwidth path of SGMV for short segments (decode-shaped batches), gfx950.
//
// When every request brings its own adapter the per-segment product is a
// matrix-vector product and the operator is bound by streaming the adapter
// weights from HBM (last paragraph of the paper's SGMV section: "totally
// IO-bound", no matrix units).  These kernels therefore use the vector ALUs
// only and are organised around keeping as many 128-bit weight loads in flight
// as possible:
//
//   shrink  one workgroup per (segment, k-slice): split-K over h_in (the paper's
//           kernel-schedule paragraph uses Split-K for the thin output too).
//           Every lane issues all of its weight loads before it consumes any,
//           accumulates eight rank columns in fp32, then the lanes are summed
//           with a transposing butterfly and the waves through LDS.  Each
//           slice writes its partial sums to the workspace; nothing is
//           accumulated with atomics, so results are deterministic.  The
//           consumer (expand, or the small reduce kernel) adds the slices in
//           a fixed order -- this replaces the grid synchronisation and
//           cross-block reduction of the paper's schedule.
//   expand  one workgroup per (segment, column block): the weight is split
//           along the output features (same as the paper's expand schedule).
//           The r-wide v rows are summed from the split-K partials into LDS
//           while the B_i loads are already in flight; y is read, updated in
//           fp32 and rounded once.
//
// The segment lookup (row range and weight pointers) is resolved once per
// workgroup from wave-uniform values.
#include <type_traits>

#include "device_common.h"
#include "launch.h"

namespace sgmv {

// ---------------------------------------------------------------- shrink
//
// grid = (n_segs, ksplit).  Slice s covers k in [s*kslice, min(h_in, (s+1)*kslice)).
// The slice of A_i is one contiguous run of kslice*R elements; 128-bit chunk q
// of it holds row k = q / LPR, columns (q % LPR)*8 .. +7, LPR = R/8.
// partials is [ksplit][n_tokens][R] fp32.
template <class DT, int R, int NT, int U, int RB>
__global__ __launch_bounds__(NT) void shrink_vector_kernel(
    const uint16_t* __restrict__ x, const uint16_t* const* __restrict__ A_ptrs,
    const int32_t* __restrict__ seg_starts, float* __restrict__ partials, int h_in, int kslice,
    int n_tokens, long long layer_off) {
  constexpr int LPR = R / 8;
  constexpr int NW = NT / 64;
  static_assert(NT % 64 == 0 && NT % LPR == 0, "bad workgroup size");
  static_assert(NT >= RB * R, "write-out needs one thread per (row, column)");
  __shared__ __align__(16) uint16_t xs[RB][kMaxKSlice];
  __shared__ float red[NW][RB][R];

  const int seg = blockIdx.x, s = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int lo = seg_starts[seg], hi = seg_starts[seg + 1];
  if (lo >= hi) return;
  const uint16_t* A = A_ptrs[seg];
  if (A == nullptr) return;
  const int k0 = s * kslice;
  const int klen = min(h_in, k0 + kslice) - k0;
  if (klen <= 0) return;
  A += layer_off + (long long)k0 * R;
  const int nchunks = klen * LPR;
  const int cpr = klen >> 3;  // 128-bit chunks per x row slice

  for (int row0 = lo; row0 < hi; row0 += RB) {
    const int nrows = min(RB, hi - row0);
    float acc[RB][8];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[rb][e] = 0.f;

    if (row0 != lo) __syncthreads();  // xs / red are reused

    for (int base = 0; base < nchunks; base += NT * U) {
      uint4 a[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int q = base + u * NT + tid;
        a[u] = (q < nchunks) ? load128_stream(A + (long long)q * 8) : make_uint4(0, 0, 0, 0);
      }
      if (base == 0) {
        // stage this row block's slice of x while the weight loads are in flight
        for (int idx = tid; idx < nrows * cpr; idx += NT) {
          const int rr = idx / cpr, c = idx - rr * cpr;
          store128(&xs[rr][c * 8], load128(x + (long long)(row0 + rr) * h_in + k0 + c * 8));
        }
        __syncthreads();
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int q = base + u * NT + tid;
        if (q < nchunks) {
          const int kk = q / LPR;
          float af[8];
          unpack8<DT>(a[u], af);
#pragma unroll
          for (int rb = 0; rb < RB; ++rb) {
            if (rb < nrows) {
              const float xv = decode1<DT>(xs[rb][kk]);
#pragma unroll
              for (int e = 0; e < 8; ++e) acc[rb][e] = fmaf(xv, af[e], acc[rb][e]);
            }
          }
        }
      }
    }

    // lanes -> one value per column, waves -> LDS
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      if (rb < nrows) {
        int e;
        const float d = reduce_lanes8<LPR>(acc[rb], lane, e);
        if (lane < R) red[wave][rb][(lane % LPR) * 8 + e] = d;
      }
    }
    __syncthreads();
    if (tid < nrows * R) {
      const int rb = tid / R, j = tid - rb * R;
      float sum = red[0][rb][j];
#pragma unroll
      for (int w = 1; w < NW; ++w) sum += red[w][rb][j];
      partials[((long long)s * n_tokens + row0 + rb) * R + j] = sum;
    }
  }
}

// v[row][j] += sum over slices of partials[s][row][j], slices in ascending order.
// grid = (n_segs, chunks): the chunk dimension strides over the segment's elements,
// four per thread, up to sixteen slices' loads in flight; rows of segments without an
// adapter are left alone.
template <int R>
__global__ __launch_bounds__(256) void shrink_reduce_kernel(
    float* __restrict__ v, const float* __restrict__ partials,
    const uint16_t* const* __restrict__ A_ptrs, const int32_t* __restrict__ seg_starts, int ksplit,
    int n_tokens) {
  const int seg = blockIdx.x;
  const int lo = seg_starts[seg], hi = seg_starts[seg + 1];
  if (lo >= hi || A_ptrs[seg] == nullptr) return;
  const long long first = (long long)lo * R, count = (long long)(hi - lo) * R;  // multiples of 4
  const long long pstride = (long long)n_tokens * R;
  for (long long i = ((long long)blockIdx.y * blockDim.x + threadIdx.x) * 4; i < count;
       i += (long long)gridDim.y * blockDim.x * 4) {
    float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
    float4 cur = *reinterpret_cast<const float4*>(v + first + i);  // in flight with the first batch
    // SB slices' loads in flight together, added in order
    auto add_slices = [&](auto sb_tag) {
      constexpr int SB = decltype(sb_tag)::value;
      for (int s0 = 0; s0 < ksplit; s0 += SB) {
        float4 q[SB];
#pragma unroll
        for (int j = 0; j < SB; ++j)
          q[j] = *reinterpret_cast<const float4*>(partials + (long long)min(s0 + j, ksplit - 1) * pstride + first + i);
#pragma unroll
        for (int j = 0; j < SB; ++j) {
          if (s0 + j < ksplit) {
            sum.x += q[j].x; sum.y += q[j].y; sum.z += q[j].z; sum.w += q[j].w;
          }
        }
      }
    };
    if (ksplit <= 4)
      add_slices(std::integral_constant<int, 4>{});
    else
      add_slices(std::integral_constant<int, 16>{});
    float4* dst = reinterpret_cast<float4*>(v + first + i);
    cur.x += sum.x; cur.y += sum.y; cur.z += sum.z; cur.w += sum.w;
    *dst = cur;
  }
}

// ---------------------------------------------------------------- expand
//
// grid = (n_segs, ceil(h_out / (NT*8))).  A lane owns eight consecutive output
// columns.  v_parts is [nparts][n_tokens][R] fp32; the rows' v is the sum of the
// parts in ascending order (nparts = 1 for a caller-supplied v).
// A_ptrs may be nullptr (stand-alone expand); when given, a segment whose A
// pointer is NULL is skipped like one whose B pointer is NULL.
// BY_ROW: grid = (rows of the batch rounded up to a multiple of eight, column strips): a
// workgroup serves one row and looks the row's segment up (n_segs of them), so that a small
// batch of long segments still fills the chip; blockIdx.x % 8, the XCD a workgroup lands on,
// takes a run of consecutive rows, which then find their segment's weights in one L2.
template <class DT, int R, int NT, int RB, bool BY_ROW>
__global__ __launch_bounds__(NT) void expand_vector_kernel(
    uint16_t* __restrict__ y, const float* __restrict__ v_parts, int nparts,
    const uint16_t* const* __restrict__ A_ptrs, const uint16_t* const* __restrict__ B_ptrs,
    const int32_t* __restrict__ seg_starts, int h_out, int n_tokens, long long layer_off,
    float scale, int n_segs) {
  constexpr int JC = R < 16 ? R : 16;  // weight rows held in registers at a time
  __shared__ float vs[RB][R];

  const int tid = threadIdx.x;
  int seg = blockIdx.x, lo, hi;
  if constexpr (BY_ROW) {
    const int row = ((int)blockIdx.x & 7) * ((int)gridDim.x >> 3) + ((int)blockIdx.x >> 3);
    if (row >= n_tokens) return;
    seg = segment_of_row(seg_starts, n_segs, row, tid & 63);
    if (seg >= n_segs) return;  // a row behind the last segment end
    lo = row;
    hi = row + 1;
  } else {
    lo = seg_starts[seg];
    hi = seg_starts[seg + 1];
  }
  if (lo >= hi) return;
  const uint16_t* B = B_ptrs[seg];
  if (B == nullptr) return;
  if (A_ptrs != nullptr && A_ptrs[seg] == nullptr) return;
  const int c0 = (blockIdx.y * NT + tid) * 8;
  const bool active = c0 < h_out;
  B += layer_off + c0;

  for (int row0 = lo; row0 < hi; row0 += RB) {
    const int nrows = min(RB, hi - row0);

    // first weight rows: issue before waiting for v
    uint4 b[JC];
#pragma unroll
    for (int j = 0; j < JC; ++j)
      b[j] = active ? load128_stream(B + (long long)j * h_out) : make_uint4(0, 0, 0, 0);
    uint4 yq[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
      if (active && rb < nrows) yq[rb] = load128(y + (long long)(row0 + rb) * h_out + c0);

    if (row0 != lo) __syncthreads();  // vs is reused
    for (int idx = tid; idx < nrows * R; idx += NT) {
      const int rr = idx / R, j = idx - rr * R;
      const float* src = v_parts + (long long)(row0 + rr) * R + j;
      float sum = src[0];
      for (int s = 1; s < nparts; ++s) sum += src[(long long)s * n_tokens * R];
      vs[rr][j] = sum;
    }
    __syncthreads();

    float acc[RB][8];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[rb][e] = 0.f;

#pragma unroll
    for (int jc = 0; jc < R; jc += JC) {
      if (jc != 0) {
#pragma unroll
        for (int j = 0; j < JC; ++j)
          b[j] = active ? load128_stream(B + (long long)(jc + j) * h_out) : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int j = 0; j < JC; ++j) {
        float bf[8];
        unpack8<DT>(b[j], bf);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
          if (rb < nrows) {
            const float vj = vs[rb][jc + j];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[rb][e] = fmaf(vj, bf[e], acc[rb][e]);
          }
        }
      }
    }

    if (active) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        if (rb < nrows) {
          float yf[8];
          unpack8<DT>(yq[rb], yf);
          uint4 out;
          out.x = pack2<DT>(yf[0] + scale * acc[rb][0], yf[1] + scale * acc[rb][1]);
          out.y = pack2<DT>(yf[2] + scale * acc[rb][2], yf[3] + scale * acc[rb][3]);
          out.z = pack2<DT>(yf[4] + scale * acc[rb][4], yf[5] + scale * acc[rb][5]);
          out.w = pack2<DT>(yf[6] + scale * acc[rb][6], yf[7] + scale * acc[rb][7]);
          store128(y + (long long)(row0 + rb) * h_out + c0, out);
        }
      }
    }
  }
}

// The same product with the weight rows of B_i divided among the four waves of a workgroup, for
// ranks from 32 on: grid = (items, ceil(h_out / 512)), a lane owns eight consecutive columns as
// above and wave w the weight rows w R/4 .. (w+1) R/4 - 1, so that all R rows of a strip are in
// flight at once (one memory round trip instead of R/16); waves 1..3 hand their partial sums to
// wave 0 through LDS, which adds them in wave order and to y.
template <class DT, int R, int RB, bool BY_ROW>
__global__ __launch_bounds__(256) void expand_split_kernel(
    uint16_t* __restrict__ y, const float* __restrict__ v_parts, int nparts,
    const uint16_t* const* __restrict__ A_ptrs, const uint16_t* const* __restrict__ B_ptrs,
    const int32_t* __restrict__ seg_starts, int h_out, int n_tokens, long long layer_off,
    float scale, int n_segs) {
  constexpr int NT = 256, NW = 4, JW = R / NW;  // weight rows per wave
  static_assert(R % NW == 0 && JW >= 2 && JW <= 16, "rank out of range for the split expand");
  __shared__ float vs[RB][R];
  __shared__ __align__(16) float red[NW - 1][RB][64 * 8];

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
  if (lo >= hi) return;
  const uint16_t* B = B_ptrs[seg];
  if (B == nullptr) return;
  if (A_ptrs != nullptr && A_ptrs[seg] == nullptr) return;
  const int c0 = (blockIdx.y * 64 + lane) * 8;
  const bool active = c0 < h_out;
  B += layer_off + (long long)wave * JW * h_out + c0;

  for (int row0 = lo; row0 < hi; row0 += RB) {
    const int nrows = min(RB, hi - row0);
    uint4 b[JW];
#pragma unroll
    for (int j = 0; j < JW; ++j)
      b[j] = active ? load128_stream(B + (long long)j * h_out) : make_uint4(0, 0, 0, 0);
    uint4 yq[RB];
    if (wave == 0) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        if (active && rb < nrows) yq[rb] = load128(y + (long long)(row0 + rb) * h_out + c0);
    }

    if (row0 != lo) __syncthreads();  // vs and red are reused
    for (int idx = tid; idx < nrows * R; idx += NT) {
      const int rr = idx / R, j = idx - rr * R;
      const float* src = v_parts + (long long)(row0 + rr) * R + j;
      float sum = src[0];
      for (int s = 1; s < nparts; ++s) sum += src[(long long)s * n_tokens * R];
      vs[rr][j] = sum;
    }
    __syncthreads();

    float acc[RB][8];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[rb][e] = 0.f;
#pragma unroll
    for (int j = 0; j < JW; ++j) {
      float bf[8];
      unpack8<DT>(b[j], bf);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        if (rb < nrows) {
          const float vj = vs[rb][wave * JW + j];
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[rb][e] = fmaf(vj, bf[e], acc[rb][e]);
        }
      }
    }
    if (wave != 0) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        if (rb < nrows) {
          float* dst = &red[wave - 1][rb][lane * 8];
          *reinterpret_cast<float4*>(dst) = make_float4(acc[rb][0], acc[rb][1], acc[rb][2], acc[rb][3]);
          *reinterpret_cast<float4*>(dst + 4) = make_float4(acc[rb][4], acc[rb][5], acc[rb][6], acc[rb][7]);
        }
      }
    }
    __syncthreads();
    if (wave == 0 && active) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        if (rb < nrows) {
#pragma unroll
          for (int w = 0; w < NW - 1; ++w) {
            const float4 p0 = *reinterpret_cast<const float4*>(&red[w][rb][lane * 8]);
            const float4 p1 = *reinterpret_cast<const float4*>(&red[w][rb][lane * 8 + 4]);
            acc[rb][0] += p0.x; acc[rb][1] += p0.y; acc[rb][2] += p0.z; acc[rb][3] += p0.w;
            acc[rb][4] += p1.x; acc[rb][5] += p1.y; acc[rb][6] += p1.z; acc[rb][7] += p1.w;
          }
          float yf[8];
          unpack8<DT>(yq[rb], yf);
          uint4 out;
          out.x = pack2<DT>(yf[0] + scale * acc[rb][0], yf[1] + scale * acc[rb][1]);
          out.y = pack2<DT>(yf[2] + scale * acc[rb][2], yf[3] + scale * acc[rb][3]);
          out.z = pack2<DT>(yf[4] + scale * acc[rb][4], yf[5] + scale * acc[rb][5]);
          out.w = pack2<DT>(yf[6] + scale * acc[rb][6], yf[7] + scale * acc[rb][7]);
          store128(y + (long long)(row0 + rb) * h_out + c0, out);
        }
      }
    }
  }
}

// ---------------------------------------------------------------- launchers

template <class DT, int R>
static hipError_t launch_shrink_t(const ShrinkArgs& a, hipStream_t st) {
  constexpr int NT = 256, U = 8, RB = 4;
  dim3 grid((unsigned)a.n_segs, (unsigned)a.ksplit);
  hipLaunchKernelGGL((shrink_vector_kernel<DT, R, NT, U, RB>), grid, dim3(NT), 0, st,
                     (const uint16_t*)a.x, (const uint16_t* const*)a.A_ptrs, a.seg_starts,
                     a.partials, a.h_in, a.kslice, a.n_tokens, a.layer_off);
  return hipGetLastError();
}

template <class DT>
static hipError_t launch_shrink_r(const ShrinkArgs& a, hipStream_t st) {
  switch (a.r) {
    case 8: return launch_shrink_t<DT, 8>(a, st);
    case 16: return launch_shrink_t<DT, 16>(a, st);
    case 32: return launch_shrink_t<DT, 32>(a, st);
    case 64: return launch_shrink_t<DT, 64>(a, st);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_shrink_vector(const ShrinkArgs& a, hipStream_t st) {
  return a.bf16 ? launch_shrink_r<BF16>(a, st) : launch_shrink_r<F16>(a, st);
}

hipError_t launch_shrink_reduce(float* v, const ShrinkArgs& a, hipStream_t st) {
  const long long longest = (long long)(a.max_seg_len > 0 ? a.max_seg_len : a.n_tokens) * a.r;
  long long chunks = (longest + 1023) / 1024;  // 256 threads x 4 elements
  if (chunks > 64) chunks = 64;
  if (chunks < 1) chunks = 1;
  dim3 grid((unsigned)a.n_segs, (unsigned)chunks);
  const uint16_t* const* ap = (const uint16_t* const*)a.A_ptrs;
  switch (a.r) {
    case 8: hipLaunchKernelGGL(shrink_reduce_kernel<8>, grid, dim3(256), 0, st, v, a.partials, ap, a.seg_starts, a.ksplit, a.n_tokens); break;
    case 16: hipLaunchKernelGGL(shrink_reduce_kernel<16>, grid, dim3(256), 0, st, v, a.partials, ap, a.seg_starts, a.ksplit, a.n_tokens); break;
    case 32: hipLaunchKernelGGL(shrink_reduce_kernel<32>, grid, dim3(256), 0, st, v, a.partials, ap, a.seg_starts, a.ksplit, a.n_tokens); break;
    case 64: hipLaunchKernelGGL(shrink_reduce_kernel<64>, grid, dim3(256), 0, st, v, a.partials, ap, a.seg_starts, a.ksplit, a.n_tokens); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <class DT, int R, int NT>
static hipError_t launch_expand_t(const ExpandArgs& a, hipStream_t st) {
  constexpr int RB = 4;
  const unsigned strips = (unsigned)((a.h_out + NT * 8 - 1) / (NT * 8));
  if (a.by_rows) {
    hipLaunchKernelGGL((expand_vector_kernel<DT, R, NT, 1, true>), dim3((unsigned)((a.n_tokens + 7) / 8 * 8), strips),
                       dim3(NT), 0, st, (uint16_t*)a.y, a.v_parts, a.nparts, (const uint16_t* const*)a.A_ptrs,
                       (const uint16_t* const*)a.B_ptrs, a.seg_starts, a.h_out, a.n_tokens, a.layer_off, a.scale,
                       a.n_segs);
    return hipGetLastError();
  }
  hipLaunchKernelGGL((expand_vector_kernel<DT, R, NT, RB, false>), dim3((unsigned)a.n_segs, strips), dim3(NT), 0, st,
                     (uint16_t*)a.y, a.v_parts, a.nparts, (const uint16_t* const*)a.A_ptrs,
                     (const uint16_t* const*)a.B_ptrs, a.seg_starts, a.h_out, a.n_tokens,
                     a.layer_off, a.scale, a.n_segs);
  return hipGetLastError();
}

template <class DT, int R>
static hipError_t launch_expand_split(const ExpandArgs& a, hipStream_t st) {
  if constexpr (R >= 32) {
    const unsigned strips = (unsigned)((a.h_out + 511) / 512);
    if (a.by_rows) {
      hipLaunchKernelGGL((expand_split_kernel<DT, R, 1, true>), dim3((unsigned)((a.n_tokens + 7) / 8 * 8), strips), dim3(256),
                         0, st, (uint16_t*)a.y, a.v_parts, a.nparts, (const uint16_t* const*)a.A_ptrs,
                         (const uint16_t* const*)a.B_ptrs, a.seg_starts, a.h_out, a.n_tokens, a.layer_off, a.scale,
                         a.n_segs);
    } else {
      hipLaunchKernelGGL((expand_split_kernel<DT, R, 4, false>), dim3((unsigned)a.n_segs, strips), dim3(256), 0, st,
                         (uint16_t*)a.y, a.v_parts, a.nparts, (const uint16_t* const*)a.A_ptrs,
                         (const uint16_t* const*)a.B_ptrs, a.seg_starts, a.h_out, a.n_tokens, a.layer_off, a.scale,
                         a.n_segs);
    }
    return hipGetLastError();
  } else {
    return hipErrorInvalidValue;
  }
}

template <class DT, int R>
static hipError_t launch_expand_nt(const ExpandArgs& a, hipStream_t st) {
  switch (a.threads) {
    case kExpandSplit: return launch_expand_split<DT, R>(a, st);
    case 64: return launch_expand_t<DT, R, 64>(a, st);
    case 128: return launch_expand_t<DT, R, 128>(a, st);
    case 256: return launch_expand_t<DT, R, 256>(a, st);
  }
  return hipErrorInvalidValue;
}

template <class DT>
static hipError_t launch_expand_r(const ExpandArgs& a, hipStream_t st) {
  switch (a.r) {
    case 8: return launch_expand_nt<DT, 8>(a, st);
    case 16: return launch_expand_nt<DT, 16>(a, st);
    case 32: return launch_expand_nt<DT, 32>(a, st);
    case 64: return launch_expand_nt<DT, 64>(a, st);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_expand_vector(const ExpandArgs& a, hipStream_t st) {
  return a.bf16 ? launch_expand_r<BF16>(a, st) : launch_expand_r<F16>(a, st);
}

}  // namespace sgmv
