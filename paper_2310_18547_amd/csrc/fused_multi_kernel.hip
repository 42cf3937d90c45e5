// Several single-row LoRA add-ons of one shape in ONE launch, gfx950.
//
// A transformer layer applies LoRA to every dense projection, and the paper
// notes that the segment indices stay the same for all of these add-ons of a
// model invocation.  The projections that read the same activations (query /
// key / value, or gate / up) are independent of each other, so their add-ons
// can share a launch.  A single add-on moves too little data to hide its fixed
// costs (launch, first-load latency, the hand-off of the Split-K partial sums
// between workgroups); here a workgroup works through several add-ons in turn
// and keeps the NEXT one's loads in flight while it reduces, exchanges and
// finishes the current one, so HBM stays busy through the phases in which a
// single add-on leaves it idle.
//
// Work split: S * n_segs * Z workgroups.  Workgroup (s, seg, z) serves k-slice s /
// column-slice s of segment seg for the projections z, z + Z, z + 2 Z, ...
// (the host launches Z = 1: one workgroup per (slice, segment) walks all
// projections; launches small enough for all workgroups to be resident side by
// side take the plain kernel in fused_kernel.hip with one projection each).
// Its work items are (row of the segment, projection); an item is exactly the
// work of one workgroup of the single add-on kernel, with the same arithmetic (only the
// number of lane groups that share the expand's weight rows may differ, so results
// agree with a separate call up to the order of the fp32 additions).
//
// Software pipeline.  The shrink of item i+1 runs BEFORE the expand of item i:
// item i+1's partial sums are published before item i's are collected, so the
// other workgroups' sums of item i have had a whole step to arrive and the poll
// for them normally succeeds at once.  Two register sets for the shrink operands
// (x, A slice) and two for the expand operands (B slice, y) alternate; a set is
// refilled with the loads of the item two steps ahead as soon as the step that
// read it is done, so about one item's worth of loads is always in flight.
//
// The per-projection pointers (x, y and the segment's A / B pointers) are put
// into LDS once at the start, so that stepping to the next item costs no
// dependent global load.  A projection whose A or B pointer is NULL for this
// segment is skipped by all S workgroups alike.
#include <type_traits>

#include "device_common.h"
#include "exchange.h"
#include "launch.h"
#include "trace.h"


namespace sgmv {

__device__ __forceinline__ unsigned long long uniform64(unsigned long long v) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return ((unsigned long long)hi << 32) | lo;
}

// The host guarantees kslice * R / 8 <= 2048 (the A slice is one batch of loads) and
// cslice / 8 <= 256 / G (the column slice is one pass).
//   exch   [n_proj][S][n_tokens][R] 64-bit words {fp32 value (high), tag (low)}
template <class DT, int R, int G>
__global__ __launch_bounds__(320) void add_lora_fused_multi_kernel(
    const int32_t* __restrict__ seg_starts, int kslice, int cslice, int h_in, int h_out, int n_tokens,
    int S, int n_proj, long long offA, long long offB, unsigned long long* exch,
    unsigned long long* header, float scale, int spin_limit, int n_segs, int Z, FusedTable tab) {
  constexpr int NT = 256, NW = 4, U = 8;
  constexpr int LPR = R / 8;
  constexpr int CPW = NT / G;  // 8-column chunks of the column slice
  constexpr int JL = R / G;    // weight rows per lane in the expand phase
  constexpr int P = kMaxProjections;
  static_assert(JL >= 1 && JL <= 8, "bad lane-group count");
  // two lane groups: neighbouring lanes, summed with a cross-lane move; more: whole waves per
  // group, summed through LDS (as in add_lora_fused_kernel, where the reasons are given)
  constexpr bool INTRA = G == 2;

  __shared__ __align__(16) uint16_t xs[kMaxKSlice];
  __shared__ float red[NW][R];
  __shared__ float vs[R];
  __shared__ int vs_complete;  // 0: a slice of the item never arrived, its row of y stays as it is
  __shared__ __align__(16) float ex[(G > 2 ? (G - 1) : 1) * CPW * 8];
  __shared__ unsigned long long ptr_x[P], ptr_y[P], ptr_a[P], ptr_b[P];
  __shared__ uint32_t mine;  // bit p: projection p is this workgroup's and has both pointers set

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  SGMV_TRACE_DECL
  SGMV_TRACE_POINT(0);
  // grid (segments of a row, S, rows of segments x Z): blockIdx.x is the fastest-varying part of
  // the linear id by which workgroups are dealt to the XCDs, so the S workgroups that exchange
  // partial sums run on one XCD and start together
  const int n_workgroups = (int)(gridDim.x * gridDim.y * gridDim.z);
  const int zstep = Z, s = blockIdx.y;
  const int row = Z == 1 ? (int)blockIdx.z
                         : __builtin_amdgcn_readfirstlane((int)(((float)blockIdx.z + 0.5f) / (float)Z));
  const int z = (int)blockIdx.z - row * Z;
  const int seg = row * gridDim.x + blockIdx.x;
  if (seg >= n_segs) {  // the grid is padded to whole rows of segments
    if (wave == 0) leave_launch_idle(header, n_workgroups, lane);
    return;
  }
  const int lo = seg_starts[seg], hi = seg_starts[seg + 1];
  if (lo >= hi || z >= n_proj) {
    if (wave == 0) leave_launch_idle(header, n_workgroups, lane);
    return;
  }
  // The first projection's pointers come through scalar loads (one round trip, as in the
  // single add-on kernel) so that its loads can be issued at once; the pointers of all
  // projections go into LDS meanwhile: one lane per projection, all lanes' loads in parallel.
  const uint16_t* const x_first = reinterpret_cast<const uint16_t*>(tab.x[z]);
  uint16_t* const y_first = reinterpret_cast<uint16_t*>(tab.y[z]);
  // (read through the constant address space: a wave-uniform address then takes the scalar
  // path, one short round trip, and the buffer resources built from the values are scalar)
  typedef const __attribute__((address_space(4))) unsigned long long* const_u64_ptr;
  const uint16_t* const a_first = reinterpret_cast<const uint16_t*>(
      ((const_u64_ptr) reinterpret_cast<unsigned long long>(tab.A_ptrs[z]))[seg]);
  const uint16_t* const b_first = reinterpret_cast<const uint16_t*>(
      ((const_u64_ptr) reinterpret_cast<unsigned long long>(tab.B_ptrs[z]))[seg]);
  const bool first_ok = a_first != nullptr && b_first != nullptr;
  // run by the exchange wave, which has no bulk loads in flight to wait for
  auto stage_pointers = [&]() {
    unsigned long long xa = 0ull, ya = 0ull, ap = 0ull, bp = 0ull;
#pragma unroll
    for (int p = 0; p < P; ++p) {  // selects from the by-value table, no memory access
      if (lane == p) {
        xa = reinterpret_cast<unsigned long long>(tab.x[p]);
        ya = reinterpret_cast<unsigned long long>(tab.y[p]);
        ap = reinterpret_cast<unsigned long long>(tab.A_ptrs[p]);
        bp = reinterpret_cast<unsigned long long>(tab.B_ptrs[p]);
      }
    }
    bool take = false;
    if (lane < n_proj) {
      const unsigned long long a = reinterpret_cast<const unsigned long long*>(ap)[seg];
      const unsigned long long b = reinterpret_cast<const unsigned long long*>(bp)[seg];
      ptr_x[lane] = xa;
      ptr_y[lane] = ya;
      ptr_a[lane] = a;
      ptr_b[lane] = b;
      take = a != 0ull && b != 0ull && lane >= z && (lane - z) % zstep == 0;
    }
    const unsigned long long votes = __ballot(take);
    if (lane == 0) mine = (uint32_t)votes;
  };

  const int k0 = s * kslice;
  const int klen = max(0, min(h_in, k0 + kslice) - k0);
  const int nchunks = klen * LPR;
  const int col_lo = min(h_out, s * cslice);
  const int ncols = max(0, min(h_out, col_lo + cslice) - col_lo);
  const long long stride = (long long)n_tokens * R;

  // Work items in order: rows of the segment, and for each row this workgroup's projections
  // (the set bits of `mine`, ascending).  Every wave walks the same sequence, with scalars only.
  struct Item {
    int row;
    uint32_t left;  // projections of this row still to do, the lowest set bit being the current one
  };
  auto item_p = [](const Item& it) { return __builtin_ctz(it.left); };
  if (wave == NW) {
    // ============================================================ exchange wave
    const uint32_t tag = launch_tag(header);
    stage_pointers();
    lds_barrier();  // (p) pointers staged
    bool timed_out = false;
    SGMV_TRACE_POINT(4);
    const uint32_t all = __builtin_amdgcn_readfirstlane(mine);
    auto valid = [&](const Item& it) { return all != 0u && it.row < hi; };
    auto next = [&](Item it) {
      it.left &= it.left - 1u;
      if (it.left == 0u) {
        it.left = all;
        ++it.row;
      }
      return it;
    };
    auto words = [&](const Item& it) {
      return exch + (long long)item_p(it) * S * stride + (long long)it.row * R;
    };
    // add the four waves' shrink sums of an item and publish them
    auto publish = [&](const Item& it) {
      lds_barrier();  // (b) xs filled
      lds_barrier();  // (c) red filled
      if (lane < R) {
        float sum = red[0][lane];
#pragma unroll
        for (int w = 1; w < NW; ++w) sum += red[w][lane];
        const unsigned long long word = ((unsigned long long)__float_as_uint(sum) << 32) | tag;
        __hip_atomic_store(words(it) + (long long)s * stride + lane, word, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
      }
    };
    // collect all S slices of an item, ascending (only the R lanes that own an element poll:
    // idle lanes polling the same words would multiply the traffic on them)
    auto collect = [&](const Item& it) {
      bool item_timed_out = false;
      if (lane < R) {
        const float sum = collect_slices(words(it) + lane, stride, S, tag, spin_limit, item_timed_out);
        vs[lane] = sum;
      }
      item_timed_out = __any(item_timed_out);
      timed_out = timed_out || item_timed_out;
      if (lane == 0) vs_complete = item_timed_out ? 0 : 1;
      lds_barrier();               // (e) vs filled
      if (G > 1 && !INTRA) lds_barrier();    // (g) ex filled
    };
    // the shrink runs one item ahead of the expand: item i+1 is published before item i is
    // collected, so the other workgroups' sums of item i have had a whole step to arrive
    Item it_e;
    it_e.row = lo;
    it_e.left = all;
    Item it_s = it_e;
    if (valid(it_s)) {
      publish(it_s);
      it_s = next(it_s);
    }
    while (valid(it_e)) {
      if (valid(it_s)) {
        publish(it_s);
        it_s = next(it_s);
      }
      collect(it_e);
      it_e = next(it_e);
    }
    if (timed_out)
      raise_timeout(header);
    leave_launch(header, n_workgroups, tag, lane);
    SGMV_TRACE_POINT(7);
    SGMV_TRACE_FLUSH(lane == 0, 4, 7);
    return;
  }

  // ================================================================ stream waves
  const int cpr = klen >> 3;                          // 128-bit chunks in one x row slice
  const int cg = INTRA ? tid % G : tid / CPW;         // lane group
  const int cc = INTRA ? tid / G : tid - cg * CPW;    // chunk within the column slice
  const uint32_t b_row0 = (uint32_t)(cg * JL) * (uint32_t)h_out * 2u;
  const uint32_t row_bytes_out = (uint32_t)h_out * 2u;
  const bool col_active = cc * 8 < ncols;

  struct ARegs {  // what the shrink of an item reads
    uint4 xr;
    uint4 a[U];
  };
  struct BRegs {  // what the expand of an item reads
    uint4 yq;
    uint4 b[JL];
  };
  auto issue_a_at = [&](ARegs& r, int row, const uint16_t* xp, const uint16_t* A) {
    const __amdgpu_buffer_rsrc_t rX = make_buffer(xp + (long long)row * h_in + k0, (uint32_t)klen * 2u);
    const __amdgpu_buffer_rsrc_t rA = make_buffer(A + offA + (long long)k0 * R, (uint32_t)nchunks * 16u);
    r.xr = buffer_load128(rX, tid < cpr ? (uint32_t)tid * 16u : kOutOfRange);
#pragma unroll
    for (int u = 0; u < U; ++u) r.a[u] = buffer_load128(rA, (uint32_t)(u * NT + tid) * 16u);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto issue_b_at = [&](BRegs& r, int row, const uint16_t* yp, const uint16_t* B) {
    const __amdgpu_buffer_rsrc_t rB = make_buffer(
        B + offB + col_lo, ncols > 0 ? (uint32_t)((long long)(R - 1) * h_out + ncols) * 2u : 0u);
    const __amdgpu_buffer_rsrc_t rY = make_buffer(yp + (long long)row * h_out + col_lo, (uint32_t)ncols * 2u);
#pragma unroll
    for (int j = 0; j < JL; ++j)
      r.b[j] = buffer_load128(rB, col_active ? b_row0 + (uint32_t)j * row_bytes_out + (uint32_t)cc * 16u : kOutOfRange);
    r.yq = buffer_load128(rY, (cg == 0 && col_active) ? (uint32_t)cc * 16u : kOutOfRange);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto issue_a = [&](ARegs& r, const Item& it) {
    const int pp = item_p(it);
    issue_a_at(r, it.row, reinterpret_cast<const uint16_t*>(uniform64(ptr_x[pp])),
               reinterpret_cast<const uint16_t*>(uniform64(ptr_a[pp])));
  };
  auto issue_b = [&](BRegs& r, const Item& it) {
    const int pp = item_p(it);
    issue_b_at(r, it.row, reinterpret_cast<const uint16_t*>(uniform64(ptr_y[pp])),
               reinterpret_cast<const uint16_t*>(uniform64(ptr_b[pp])));
  };
  // shrink and expand of one item (the arithmetic of the single add-on kernel)
  auto shrink = [&](const ARegs& r) {
    SGMV_TRACE_POINT(9);
    store128(&xs[tid * 8], r.xr);  // chunks that do not exist arrive as zeros
    lds_barrier();                 // (b) xs filled
    SGMV_TRACE_POINT(2);
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int q = u * NT + tid;
      const int kk = (q / LPR) & (kMaxKSlice - 1);
      float af[8];
      unpack8<DT>(r.a[u], af);
      const float xraw = decode1<DT>(xs[kk]);
      const float xv = (q < nchunks) ? xraw : 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = fmaf(xv, af[e], acc[e]);
    }
    {
      int e;
      const float d = reduce_lanes8<LPR>(acc, lane, e);
      if (lane < R) red[wave][(lane % LPR) * 8 + e] = d;
    }
    SGMV_TRACE_POINT(3);
    lds_barrier();  // (c) red filled
  };
  auto expand = [&](const BRegs& r, const Item& it) {
    lds_barrier();  // (e) vs filled
    const bool complete = vs_complete != 0;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
    for (int j = 0; j < JL; ++j) {
      float bf[8];
      unpack8<DT>(r.b[j], bf);
      const float vj = vs[cg * JL + j];
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = fmaf(vj, bf[e], acc[e]);
    }
    if (INTRA) {
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += neighbour_lane(acc[e]);
    } else if (G > 1) {
      if (cg > 0) {
        float* dst = &ex[((cg - 1) * CPW + cc) * 8];
        *reinterpret_cast<float4*>(dst) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        *reinterpret_cast<float4*>(dst + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
      }
      lds_barrier();  // (g) ex filled
      if (cg == 0) {
#pragma unroll
        for (int g = 1; g < G; ++g) {
          const float* srcp = &ex[((g - 1) * CPW + cc) * 8];
          const float4 p0 = *reinterpret_cast<const float4*>(srcp);
          const float4 p1 = *reinterpret_cast<const float4*>(srcp + 4);
          acc[0] += p0.x; acc[1] += p0.y; acc[2] += p0.z; acc[3] += p0.w;
          acc[4] += p1.x; acc[5] += p1.y; acc[6] += p1.z; acc[7] += p1.w;
        }
      }
    }
    if (cg == 0) {
      uint16_t* yp = reinterpret_cast<uint16_t*>(uniform64(ptr_y[item_p(it)]));
      const __amdgpu_buffer_rsrc_t rY = make_buffer(yp + (long long)it.row * h_out + col_lo, (uint32_t)ncols * 2u);
      float yf[8];
      unpack8<DT>(r.yq, yf);
      uint4 out;
      out.x = pack2<DT>(yf[0] + scale * acc[0], yf[1] + scale * acc[1]);
      out.y = pack2<DT>(yf[2] + scale * acc[2], yf[3] + scale * acc[3]);
      out.z = pack2<DT>(yf[4] + scale * acc[4], yf[5] + scale * acc[5]);
      out.w = pack2<DT>(yf[6] + scale * acc[6], yf[7] + scale * acc[7]);
      buffer_store128(rY, (col_active && complete) ? (uint32_t)cc * 16u : kOutOfRange, out);
    }
  };

  ARegs a0, a1;
  BRegs b0, b1;
  if (first_ok) {
    issue_a_at(a0, lo, x_first, a_first);
    issue_b_at(b0, lo, y_first, b_first);
  }
  SGMV_TRACE_POINT(8);
  lds_barrier();  // (p) pointers staged
  SGMV_TRACE_POINT(1);
  const uint32_t all = __builtin_amdgcn_readfirstlane(mine);
  auto valid = [&](const Item& it) { return all != 0u && it.row < hi; };
  auto next = [&](Item it) {
    it.left &= it.left - 1u;
    if (it.left == 0u) {
      it.left = all;
      ++it.row;
    }
    return it;
  };
  // Four cursors over the same item sequence: the next item to expand, to shrink (one
  // ahead), and to fetch the shrink / expand operands of (two ahead of their use).  A
  // register set is refilled as soon as the step that read it is done.
  Item it_e;
  it_e.row = lo;
  it_e.left = all;
  Item it_s = it_e, it_a = it_e, it_b = it_e;
  if (valid(it_e)) {
    // (if the first projection has both pointers it is the first item, already issued)
    if (!first_ok) {
      issue_a(a0, it_a);
      issue_b(b0, it_b);
    }
    it_a = next(it_a);
    it_b = next(it_b);
    if (valid(it_a)) {
      issue_a(a1, it_a);
      it_a = next(it_a);
      issue_b(b1, it_b);
      it_b = next(it_b);
    }
    shrink(a0);
    it_s = next(it_s);
    if (valid(it_a)) {
      issue_a(a0, it_a);
      it_a = next(it_a);
    }
  }
  // one step: shrink the item after the one that is expanded, refill what was read
  auto step = [&](ARegs& a_sh, BRegs& b_ex) {
    if (valid(it_s)) {
      shrink(a_sh);
      it_s = next(it_s);
      if (valid(it_a)) {
        issue_a(a_sh, it_a);
        it_a = next(it_a);
      }
    }
    expand(b_ex, it_e);
    it_e = next(it_e);
    if (valid(it_b)) {
      issue_b(b_ex, it_b);
      it_b = next(it_b);
    }
  };
  while (valid(it_e)) {
    step(a1, b0);
    if (!valid(it_e)) break;
    step(a0, b1);
  }
  SGMV_TRACE_POINT(6);
  SGMV_TRACE_FLUSH(tid == 0, 0, 3);
  SGMV_TRACE_FLUSH(tid == 0, 6, 6);
  SGMV_TRACE_FLUSH(tid == 0, 8, 9);
}

template <class DT, int R, int G>
static hipError_t launch_multi_t(const FusedArgs& a, hipStream_t st) {
  hipLaunchKernelGGL((add_lora_fused_multi_kernel<DT, R, G>),
                     dim3((unsigned)fused_grid_x(a.n_segs), (unsigned)a.S,
                          (unsigned)(fused_grid_items(a.n_segs) / fused_grid_x(a.n_segs) * a.Z)),
                     dim3(320), 0, st, a.seg_starts, a.kslice, a.cslice, a.h_in, a.h_out, a.n_tokens, a.S,
                     a.n_proj, a.offA, a.offB, a.exch, a.header, a.scale, a.spin_limit, a.n_segs, a.Z, a.table);
  return hipGetLastError();
}

template <class DT, int R>
static hipError_t launch_multi_g(const FusedArgs& a, hipStream_t st) {
  // at most eight weight rows per lane in the expand phase: two register sets must fit
  switch (a.G) {
    case 1: if constexpr (R <= 8) return launch_multi_t<DT, R, 1>(a, st); break;
    case 2: if constexpr (R <= 16) return launch_multi_t<DT, R, 2>(a, st); break;
    case 4: if constexpr (R <= 32) return launch_multi_t<DT, R, 4>(a, st); break;
    case 8: return launch_multi_t<DT, R, 8>(a, st);
  }
  return hipErrorInvalidValue;
}

template <class DT>
static hipError_t launch_multi_r(const FusedArgs& a, hipStream_t st) {
  switch (a.r) {
    case 8: return launch_multi_g<DT, 8>(a, st);
    case 16: return launch_multi_g<DT, 16>(a, st);
    case 32: return launch_multi_g<DT, 32>(a, st);
    case 64: return launch_multi_g<DT, 64>(a, st);
  }
  return hipErrorInvalidValue;
}

// True when the launch shape fits the kernel: the A slice is one batch of loads and the
// column slice one pass.
bool fused_multi_fits(const FusedArgs& a) {
  return (long long)a.kslice * (a.r / 8) <= 2048 && a.cslice / 8 <= 256 / a.G && a.r / a.G <= 8;
}

hipError_t launch_add_lora_fused_multi(const FusedArgs& a, hipStream_t st) {
  if (!fused_multi_fits(a) || a.n_proj < 1 || a.n_proj > kMaxProjections || a.Z < 1) return hipErrorInvalidValue;
  return a.bf16 ? launch_multi_r<BF16>(a, st) : launch_multi_r<F16>(a, st);
}

}  // namespace sgmv
