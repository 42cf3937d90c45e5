// Single-launch LoRA add-on for decode-shaped batches (short segments), gfx950.
//
// The paper evaluates the add-on as two launches of the SGMV kernel (v += xA,
// then y += vB) and, inside the shrink launch, a grid synchronisation followed
// by a cross-block reduction of the Split-K partial sums.  On MI355X a kernel
// boundary costs about as much as streaming the whole batch's adapter weights
// (the operator moves ~18 MB; an empty launch is ~1.5 us), so here both steps
// run in ONE launch and the only cross-workgroup hand-off is per segment:
//
//   * S workgroups serve one segment.  Workgroup s first does the shrink of
//     k-slice s for all rows of the segment, then the expand of column-slice s.
//   * All weight loads of both phases (its A slice and its B slice) are issued
//     at the very start, A first, so the B slice streams in while the shrink
//     is computed and the partial sums are exchanged.
//   * Partial sums go to the workspace; a per-segment arrival counter
//     (release / acquire at agent scope, the L2s of the eight XCDs are not
//     coherent with each other) tells the S consumers when all slices are
//     there.  Every consumer adds the slices in the same ascending order, so
//     the result is deterministic.  The last consumer to read resets the
//     segment's counters for the next call.
//   * Producers never wait before publishing, the S workgroups of a segment
//     have consecutive ids, and workgroups are dispatched in id order, so a
//     waiting workgroup only ever waits for workgroups that are already
//     resident or next in line.  The wait is bounded all the same: after
//     spin_limit polls a workgroup raises the workspace's error word and
//     leaves, so no wave can stay in the kernel for ever.
#include "device_common.h"
#include "launch.h"

namespace sgmv {

template <int LPR>
__device__ __forceinline__ float fused_reduce_lanes8(const float (&a)[8], int lane, int& e_out) {
  constexpr int M1 = LPR, M2 = LPR * 2, M3 = LPR * 4;
  float b[4], c[2], d;
  bool up = (lane & M1) != 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float send = up ? a[i] : a[i + 4];
    float keep = up ? a[i + 4] : a[i];
    b[i] = keep + __shfl_xor(send, M1, 64);
  }
  up = (lane & M2) != 0;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    float send = up ? b[i] : b[i + 2];
    float keep = up ? b[i + 2] : b[i];
    c[i] = keep + __shfl_xor(send, M2, 64);
  }
  up = (lane & M3) != 0;
  {
    float send = up ? c[0] : c[1];
    float keep = up ? c[1] : c[0];
    d = keep + __shfl_xor(send, M3, 64);
  }
#pragma unroll
  for (int m = M3 * 2; m < 64; m <<= 1) d += __shfl_xor(d, m, 64);
  e_out = ((lane & M1) ? 4 : 0) | ((lane & M2) ? 2 : 0) | ((lane & M3) ? 1 : 0);
  return d;
}

// grid = n_segs * S workgroups of 256 threads; workgroup w serves segment w / S
// with slice index w % S.
//   partials  [S][n_tokens][R] fp32
//   counters  arrive[n_tokens], done[n_tokens] (indexed by the segment's first
//             row), then one error word; all zero between calls
// G = lane groups of the expand phase: group g multiplies weight rows
// g*R/G .. (g+1)*R/G-1; the groups are summed through LDS.
template <class DT, int R, int G, int RB>
__global__ __launch_bounds__(256) void add_lora_fused_kernel(
    uint16_t* __restrict__ y, const uint16_t* __restrict__ x,
    const uint16_t* const* __restrict__ A_ptrs, const uint16_t* const* __restrict__ B_ptrs,
    const int32_t* __restrict__ seg_starts, float* partials, unsigned* counters, int h_in,
    int h_out, int S, int kslice, int cslice, int n_tokens, long long offA, long long offB,
    float scale, int spin_limit) {
  constexpr int NT = 256, NW = 4, U = 8;
  constexpr int LPR = R / 8;
  constexpr int CPW = NT / G;  // 8-column chunks per pass
  constexpr int JL = R / G;    // weight rows per lane in the expand phase
  constexpr int XU = RB * kMaxKSlice / 8 / NT;
  static_assert(JL >= 1 && JL <= 16, "bad lane-group count");
  static_assert(NT >= RB * R, "one thread per (row, column) of a row block");

  __shared__ __align__(16) uint16_t xs[RB][kMaxKSlice];
  __shared__ float red[NW][RB][R];
  __shared__ float vs[RB][R];
  __shared__ __align__(16) float ex[(G > 1 ? (G - 1) : 1) * RB * CPW * 8];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int seg = blockIdx.x / S, s = blockIdx.x - seg * S;
  const int lo = seg_starts[seg], hi = seg_starts[seg + 1];
  if (lo >= hi) return;
  const uint16_t* A = A_ptrs[seg];
  const uint16_t* B = B_ptrs[seg];
  if (A == nullptr || B == nullptr) return;  // same decision in all S workgroups

  // ---- shrink geometry
  const int k0 = s * kslice;
  const int klen = max(0, min(h_in, k0 + kslice) - k0);
  const int nchunks = klen * LPR;
  const int cpr = klen >> 3;
  A += offA + (long long)k0 * R;
  // ---- expand geometry
  const int col_lo = s * cslice;
  const int col_hi = min(h_out, col_lo + cslice);
  const int cg = tid / CPW, cc = tid - cg * CPW;  // lane group, chunk within pass
  B += offB + (long long)(cg * JL) * h_out;

  // ---- issue everything that does not depend on another workgroup: A, x, B, y
  uint4 a[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int q = u * NT + tid;
    a[u] = (q < nchunks) ? load128_stream(A + (long long)q * 8) : make_uint4(0, 0, 0, 0);
  }
  uint4 xr[XU];
  {
    const int nrows = min(RB, hi - lo);
#pragma unroll
    for (int i = 0; i < XU; ++i) {
      const int idx = i * NT + tid;
      if (idx < nrows * cpr) {
        const int rr = idx / cpr, c = idx - rr * cpr;
        xr[i] = load128(x + (long long)(lo + rr) * h_in + k0 + c * 8);
      }
    }
  }
  uint4 b[JL];
  {
    const int c0 = col_lo + cc * 8;
#pragma unroll
    for (int j = 0; j < JL; ++j)
      b[j] = (c0 < col_hi) ? load128_stream(B + (long long)j * h_out + c0) : make_uint4(0, 0, 0, 0);
  }
  uint4 yq[RB];
  {
    const int c0 = col_lo + cc * 8;
    const int nrows = min(RB, hi - lo);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
      if (cg == 0 && c0 < col_hi && rb < nrows) yq[rb] = load128(y + (long long)(lo + rb) * h_out + c0);
  }

  // ================================================================ shrink
  for (int row0 = lo; row0 < hi; row0 += RB) {
    const int nrows = min(RB, hi - row0);
    float acc[RB][8];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[rb][e] = 0.f;

    if (row0 != lo) {
      __syncthreads();  // xs / red are reused
#pragma unroll
      for (int i = 0; i < XU; ++i) {
        const int idx = i * NT + tid;
        if (idx < nrows * cpr) {
          const int rr = idx / cpr, c = idx - rr * cpr;
          xr[i] = load128(x + (long long)(row0 + rr) * h_in + k0 + c * 8);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < XU; ++i) {
      const int idx = i * NT + tid;
      if (idx < nrows * cpr) {
        const int rr = idx / cpr, c = idx - rr * cpr;
        store128(&xs[rr][c * 8], xr[i]);
      }
    }
    __syncthreads();

    for (int base = 0; base < nchunks; base += NT * U) {
      if (base != 0 || row0 != lo) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int q = base + u * NT + tid;
          a[u] = (q < nchunks) ? load128_stream(A + (long long)q * 8) : make_uint4(0, 0, 0, 0);
        }
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

#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      if (rb < nrows) {
        int e;
        const float d = fused_reduce_lanes8<LPR>(acc[rb], lane, e);
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

  // ================================================================ hand-off
  unsigned* arrive = counters + lo;
  unsigned* done = counters + n_tokens + lo;
  unsigned* error_word = counters + 2 * (long long)n_tokens;
  __syncthreads();  // every partial of this workgroup has been stored
  if (tid == 0) {
    __hip_atomic_fetch_add(arrive, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    int polls = 0;
    while (__hip_atomic_load(arrive, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < (unsigned)S) {
      if (++polls > spin_limit) {
        __hip_atomic_store(error_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
  }
  __syncthreads();  // the acquire above now covers the whole workgroup

  // ================================================================ expand
  const int npass = (col_hi - col_lo + CPW * 8 - 1) / (CPW * 8);  // <= 0 when the slice is empty
  for (int row0 = lo; row0 < hi; row0 += RB) {
    const int nrows = min(RB, hi - row0);
    if (row0 != lo) __syncthreads();  // vs is reused
    if (tid < nrows * R) {
      const int rb = tid / R, j = tid - rb * R;
      const float* src = partials + (long long)(row0 + rb) * R + j;
      const long long stride = (long long)n_tokens * R;
      float sum = 0.f;
      for (int s0 = 0; s0 < S; s0 += 8) {
        float t[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) t[i] = (s0 + i < S) ? src[(s0 + i) * stride] : 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) sum += t[i];
      }
      vs[rb][j] = sum;
    }
    __syncthreads();
    if (row0 + RB >= hi && tid == 0) {
      // this workgroup has read everything it needs from the segment's partials
      const unsigned before = __hip_atomic_fetch_add(done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (before == (unsigned)S - 1u) {
        __hip_atomic_store(arrive, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }

    for (int pass = 0; pass < npass; ++pass) {
      const int c0 = col_lo + (pass * CPW + cc) * 8;
      const bool active = c0 < col_hi;
      if (pass != 0 || row0 != lo) {
        if (npass > 1) {
#pragma unroll
          for (int j = 0; j < JL; ++j)
            b[j] = active ? load128_stream(B + (long long)j * h_out + c0) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
          if (cg == 0 && active && rb < nrows) yq[rb] = load128(y + (long long)(row0 + rb) * h_out + c0);
      }
      float acc[RB][8];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[rb][e] = 0.f;
#pragma unroll
      for (int j = 0; j < JL; ++j) {
        float bf[8];
        unpack8<DT>(b[j], bf);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
          if (rb < nrows) {
            const float vj = vs[rb][cg * JL + j];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[rb][e] = fmaf(vj, bf[e], acc[rb][e]);
          }
        }
      }
      if (G > 1) {
        if (pass != 0) __syncthreads();  // ex is reused
        if (cg > 0) {
#pragma unroll
          for (int rb = 0; rb < RB; ++rb) {
            if (rb < nrows) {
              float* dst = &ex[(((cg - 1) * RB + rb) * CPW + cc) * 8];
              *reinterpret_cast<float4*>(dst) = make_float4(acc[rb][0], acc[rb][1], acc[rb][2], acc[rb][3]);
              *reinterpret_cast<float4*>(dst + 4) = make_float4(acc[rb][4], acc[rb][5], acc[rb][6], acc[rb][7]);
            }
          }
        }
        __syncthreads();
        if (cg == 0) {
#pragma unroll
          for (int g = 1; g < G; ++g) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
              if (rb < nrows) {
                const float* srcp = &ex[(((g - 1) * RB + rb) * CPW + cc) * 8];
                const float4 p0 = *reinterpret_cast<const float4*>(srcp);
                const float4 p1 = *reinterpret_cast<const float4*>(srcp + 4);
                acc[rb][0] += p0.x; acc[rb][1] += p0.y; acc[rb][2] += p0.z; acc[rb][3] += p0.w;
                acc[rb][4] += p1.x; acc[rb][5] += p1.y; acc[rb][6] += p1.z; acc[rb][7] += p1.w;
              }
            }
          }
        }
      }
      if (cg == 0 && active) {
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
}

// Fill kernel used to zero the workspace (a kernel rather than a memset so the
// call can be recorded into a HIP graph).
__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t* p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = 0u;
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st) {
  const size_t n = bytes / 4;
  if (n == 0) return hipSuccess;
  unsigned blocks = (unsigned)((n + 255) / 256);
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, st, (uint32_t*)p, n);
  return hipGetLastError();
}

template <class DT, int R, int G>
static hipError_t launch_fused_t(const FusedArgs& a, hipStream_t st) {
  constexpr int RB = 4;
  hipLaunchKernelGGL((add_lora_fused_kernel<DT, R, G, RB>), dim3((unsigned)(a.n_segs * a.S)),
                     dim3(256), 0, st, (uint16_t*)a.y, (const uint16_t*)a.x,
                     (const uint16_t* const*)a.A_ptrs, (const uint16_t* const*)a.B_ptrs,
                     a.seg_starts, a.partials, a.counters, a.h_in, a.h_out, a.S, a.kslice,
                     a.cslice, a.n_tokens, a.offA, a.offB, a.scale, a.spin_limit);
  return hipGetLastError();
}

template <class DT, int R>
static hipError_t launch_fused_g(const FusedArgs& a, hipStream_t st) {
  switch (a.G) {
    case 1: if constexpr (R <= 16) return launch_fused_t<DT, R, 1>(a, st); break;
    case 2: if constexpr (R <= 32) return launch_fused_t<DT, R, 2>(a, st); break;
    case 4: return launch_fused_t<DT, R, 4>(a, st);
    case 8: return launch_fused_t<DT, R, 8>(a, st);
  }
  return hipErrorInvalidValue;
}

template <class DT>
static hipError_t launch_fused_r(const FusedArgs& a, hipStream_t st) {
  switch (a.r) {
    case 8: return launch_fused_g<DT, 8>(a, st);
    case 16: return launch_fused_g<DT, 16>(a, st);
    case 32: return launch_fused_g<DT, 32>(a, st);
    case 64: return launch_fused_g<DT, 64>(a, st);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_add_lora_fused(const FusedArgs& a, hipStream_t st) {
  return a.bf16 ? launch_fused_r<BF16>(a, st) : launch_fused_r<F16>(a, st);
}

}  // namespace sgmv
