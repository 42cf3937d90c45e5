// Single-launch LoRA add-on for decode-shaped batches (short segments), gfx950.
//
// The paper evaluates the add-on as two launches of the SGMV kernel (v += xA,
// then y += vB) and, inside the shrink launch, a grid synchronisation followed
// by a cross-block reduction of the Split-K partial sums.  On MI355X a kernel
// boundary costs about as much as streaming the whole batch's adapter weights
// (the operator moves ~18 MB; an empty launch is ~1.5 us), so here both steps
// run in ONE launch and the only cross-workgroup hand-off is per segment.
//
// Work split.  S workgroups serve one segment.  Workgroup s does the shrink of
// k-slice s for all rows of the segment, then the expand of column-slice s.
// A workgroup has five waves:
//   * four STREAM waves issue every weight load of both phases at the very
//     start (x, then the A slice, then the B slice, then y) through buffer
//     resources, whose hardware range check does the predication, so the loads
//     sit back to back with no branches between them.  They multiply, reduce
//     their lanes with a transposing butterfly and leave per-wave sums in LDS;
//     later they pick the complete v rows up from LDS and finish the expand.
//     The barriers between the phases order LDS only, so a stream wave never
//     drains its outstanding B / y loads while the partial sums are exchanged.
//   * one EXCHANGE wave, which has no bulk loads in flight (vector memory
//     returns in order, so a wave that polls must not queue behind its own
//     streaming loads), publishes the workgroup's partial sums and collects
//     those of the other S-1 workgroups.
//
// Hand-off.  The L2s of the eight XCDs are not coherent with each other, so
// the exchanged words are written and read with agent-scope accesses that
// bypass them.  A partial sum travels as one 64-bit word {value, tag}; the tag
// is the workspace's generation (exchange.h), so a consumer simply polls the S
// words it needs until their tags match -- there is no separate flag, no
// ordering between separate stores to get wrong, and nothing to reset
// afterwards.  Calls that share a workspace must be stream-ordered.
//
// Every consumer adds the S slices in the same ascending order, so results are
// deterministic.  Producers never wait before publishing, the S workgroups of
// a segment have consecutive ids and workgroups are dispatched in id order, so
// a polling workgroup only waits for workgroups that are resident or next in
// line.  The wait is bounded all the same: after spin_limit polls a workgroup
// raises the workspace's error word and carries on, so no wave can stay in the
// kernel for ever.
#include <type_traits>

#include "device_common.h"
#include "exchange.h"
#include "launch.h"
#include "trace.h"


namespace sgmv {

// Body of the kernels below: workgroup of 320 threads that serves slice `s` of segment `seg`
// (the kernels derive both from blockIdx without a division).
//   exch   [S][n_tokens][R] 64-bit words {fp32 value (high), tag (low)}
//   header the workspace's generation copies, then the error flag
// G  = lane groups of the expand phase: group g multiplies weight rows
//      g*R/G .. (g+1)*R/G-1; the groups are summed through LDS.
// RB = rows handled per pass over the weights (1 when every segment is one row).
// BY_ROW: `seg` is a row of the batch, not a segment: the workgroup serves that one row and
//      looks its segment up in seg_starts (n_segs of them).
template <class DT, int R, int G, int RB, bool BY_ROW = false>
__device__ __forceinline__ void add_lora_fused_body(
    const int32_t* __restrict__ seg_starts, const uint16_t* const* __restrict__ A_ptrs,
    const uint16_t* const* __restrict__ B_ptrs, const uint16_t* __restrict__ x,
    uint16_t* __restrict__ y, int kslice, int cslice, int h_in, int h_out, int n_tokens, int S,
    long long offA, long long offB, unsigned long long* exch, unsigned long long* header,
    float scale, int spin_limit, int seg, int s, int n_segs = 0) {
  constexpr int NT = 256, NW = 4, U = 8;  // stream threads / waves, A loads per lane and batch
  constexpr int LPR = R / 8;
  constexpr int CPW = NT / G;  // 8-column chunks per pass
  constexpr int JL = R / G;    // weight rows per lane in the expand phase
  static_assert(JL >= 1 && JL <= 16, "bad lane-group count");
  static_assert(kMaxKSlice / 8 == NT, "one 128-bit x chunk per lane and row");
  // Two lane groups sit in neighbouring lanes of a wave (lane group = lane % 2) and add their
  // sums with cross-lane moves: no LDS, no barrier, 0.2 us less behind the hand-off (B = 64:
  // 6.23 -> 6.02 us).  With four or eight groups a wave's loads of B_i would fall into runs of
  // 256 or 128 bytes per weight row, which costs more than the barriers (B = 64 at rank 64:
  // 15.4 -> 16.6 us), so those keep whole waves per group and meet in LDS.
  constexpr bool INTRA = G == 2;

  __shared__ __align__(16) uint16_t xs[RB][kMaxKSlice];
  __shared__ __align__(16) float red[NW * 4][RB][R];  // per wave and row of sixteen lanes
  __shared__ float vs[RB][R];
  __shared__ int vs_complete;  // 0: a slice of this row block never arrived, its rows of y stay as they are
  __shared__ __align__(16) float ex[(G > 2 ? (G - 1) : 1) * RB * CPW * 8];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  SGMV_TRACE_DECL
  SGMV_TRACE_POINT(0);
  int lo, hi;
  const uint16_t *A, *B;
  if constexpr (BY_ROW) {
    const int found = segment_of_row(seg_starts, n_segs, seg, lane);
    lo = seg;
    hi = found < n_segs ? seg + 1 : seg;  // a row behind the last segment end: nothing to do
    A = found < n_segs ? A_ptrs[found] : nullptr;
    B = found < n_segs ? B_ptrs[found] : nullptr;
  } else {
    lo = seg_starts[seg];
    hi = seg_starts[seg + 1];
    A = A_ptrs[seg];
    B = B_ptrs[seg];
  }
  if (lo >= hi || A == nullptr || B == nullptr) {  // same decision in all S workgroups
    if (wave == 0) leave_launch_idle(header, (int)(gridDim.x * gridDim.y * gridDim.z), lane);
    return;
  }
  SGMV_TRACE_POINT(8);
  const int k0 = s * kslice;
  const int klen = max(0, min(h_in, k0 + kslice) - k0);
  const int nchunks = klen * LPR;  // 128-bit chunks in this workgroup's slice of A_i
  const int col_lo = min(h_out, s * cslice);
  const int ncols = max(0, min(h_out, col_lo + cslice) - col_lo);
  const int npass = (ncols + CPW * 8 - 1) / (CPW * 8);  // 0 when the column slice is empty

  if (wave == NW) {
    // ============================================================ exchange wave
    const uint32_t tag = launch_tag(header);
    SGMV_TRACE_POINT(9);
    const long long stride = (long long)n_tokens * R;
    // ---- shrink phase: publish this workgroup's partial sums
    for (int row0 = lo; row0 < hi; row0 += RB) {
      const int nrows = min(RB, hi - row0);
      if (row0 != lo) lds_barrier();  // (a) xs / red free
      lds_barrier();                  // (b) xs filled
      lds_barrier();                  // (c) red filled
      for (int idx = lane; idx < nrows * R; idx += 64) {
        const int rb = idx / R, j = idx - rb * R;
        float sum = red[0][rb][j];
#pragma unroll
        for (int w = 1; w < NW * 4; ++w) sum += red[w][rb][j];
        const unsigned long long word = ((unsigned long long)__float_as_uint(sum) << 32) | tag;
        __hip_atomic_store(exch + (long long)s * stride + (long long)(row0 + rb) * R + j, word,
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    SGMV_TRACE_POINT(4);
    // ---- expand phase: collect all S slices of every row, in ascending order
    bool timed_out = false;
    for (int row0 = lo; row0 < hi; row0 += RB) {
      const int nrows = min(RB, hi - row0);
      if (row0 != lo) lds_barrier();  // (d) vs / ex free
      bool block_timed_out = false;
      for (int idx = lane; idx < nrows * R; idx += 64) {
        const int rb = idx / R, j = idx - rb * R;
        const unsigned long long* src = exch + (long long)(row0 + rb) * R + j;
        const float sum = collect_slices(src, stride, S, tag, spin_limit, block_timed_out);
        vs[rb][j] = sum;
      }
      block_timed_out = __any(block_timed_out);
      timed_out = timed_out || block_timed_out;
      if (lane == 0) vs_complete = block_timed_out ? 0 : 1;
      SGMV_TRACE_POINT(5);
      lds_barrier();  // (e) vs filled
      if (G > 1 && !INTRA) {
        for (int pass = 0; pass < npass; ++pass) {
          if (pass != 0) lds_barrier();  // (f) ex free
          lds_barrier();                 // (g) ex filled
        }
      }
    }
    if (timed_out) raise_timeout(header);
    leave_launch(header, (int)(gridDim.x * gridDim.y * gridDim.z), tag, lane);
    SGMV_TRACE_POINT(7);
    SGMV_TRACE_FLUSH(lane == 0, 4, 7);
    SGMV_TRACE_FLUSH(lane == 0, 9, 9);
    return;
  }

  // ================================================================ stream waves
  const int cpr = klen >> 3;  // 128-bit chunks in one x row slice
  const __amdgpu_buffer_rsrc_t rA = make_buffer(A + offA + (long long)k0 * R, (uint32_t)nchunks * 16u);
  const int cg = INTRA ? tid % G : tid / CPW;  // lane group
  const int cc = INTRA ? tid / G : tid - cg * CPW;  // chunk within pass
  const __amdgpu_buffer_rsrc_t rB = make_buffer(
      B + offB + col_lo, ncols > 0 ? (uint32_t)((long long)(R - 1) * h_out + ncols) * 2u : 0u);
  const uint32_t b_row0 = (uint32_t)(cg * JL) * (uint32_t)h_out * 2u;
  const uint32_t row_bytes_out = (uint32_t)h_out * 2u;

  // ---- issue everything that does not depend on another workgroup: x, A, B, y
  const int nrows_first = min(RB, hi - lo);
  uint4 xr[RB];
  {
    const __amdgpu_buffer_rsrc_t rX = make_buffer(
        x + (long long)lo * h_in + k0, (uint32_t)((long long)(nrows_first - 1) * h_in + klen) * 2u);
#pragma unroll
    for (int rr = 0; rr < RB; ++rr)
      xr[rr] = buffer_load128(rX, (tid < cpr && rr < nrows_first) ? (uint32_t)(rr * h_in + tid * 8) * 2u : kOutOfRange);
  }
  uint4 a[U];
#pragma unroll
  for (int u = 0; u < U; ++u) a[u] = buffer_load128(rA, (uint32_t)(u * NT + tid) * 16u);
  __builtin_amdgcn_sched_barrier(0);  // keep x and A ahead of B and y in the memory pipe
  uint4 b[JL];
  uint4 yq[RB];
  auto issue_b_y = [&]() {
    {
      const bool active = cc * 8 < ncols;
#pragma unroll
      for (int j = 0; j < JL; ++j)
        b[j] = buffer_load128(rB, active ? b_row0 + (uint32_t)j * row_bytes_out + (uint32_t)cc * 16u : kOutOfRange);
    }
    {
      const __amdgpu_buffer_rsrc_t rY = make_buffer(
          y + (long long)lo * h_out + col_lo,
          ncols > 0 ? (uint32_t)((long long)(nrows_first - 1) * h_out + ncols) * 2u : 0u);
      const bool active = cg == 0 && cc * 8 < ncols;
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        yq[rb] = buffer_load128(rY, (active && rb < nrows_first) ? (uint32_t)rb * row_bytes_out + (uint32_t)cc * 16u : kOutOfRange);
    }
  };
  issue_b_y();
  __builtin_amdgcn_sched_barrier(0);
  SGMV_TRACE_POINT(1);

  // One row block of the shrink phase.  `first` selects the copy that uses the
  // loads issued above; it is a separate, straight-line copy so that the waits
  // in it count exactly the loads that are still needed.
  auto shrink_block = [&](int row0, auto first_tag) {
    constexpr bool first = decltype(first_tag)::value;
    const int nrows = min(RB, hi - row0);
    float acc[RB][8];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[rb][e] = 0.f;
    if (!first) {
      lds_barrier();  // (a) xs / red free
      const __amdgpu_buffer_rsrc_t rX = make_buffer(
          x + (long long)row0 * h_in + k0, (uint32_t)((long long)(nrows - 1) * h_in + klen) * 2u);
#pragma unroll
      for (int rr = 0; rr < RB; ++rr)
        xr[rr] = buffer_load128(rX, (tid < cpr && rr < nrows) ? (uint32_t)(rr * h_in + tid * 8) * 2u : kOutOfRange);
    }
    // rows and chunks that do not exist arrive as zeros, so xs is always fully defined
#pragma unroll
    for (int rr = 0; rr < RB; ++rr) store128(&xs[rr][tid * 8], xr[rr]);
    lds_barrier();  // (b) xs filled
    SGMV_TRACE_POINT(2);

    for (int base = 0; base < nchunks; base += NT * U) {
      if (!first || base != 0) {
#pragma unroll
        for (int u = 0; u < U; ++u) a[u] = buffer_load128(rA, (uint32_t)(base + u * NT + tid) * 16u);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int q = base + u * NT + tid;
        const int kk = (q / LPR) & (kMaxKSlice - 1);
        float af[8];
        unpack8<DT>(a[u], af);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
          if (RB == 1 || rb < nrows) {
            const float xraw = decode1<DT>(xs[rb][kk]);
            const float xv = (q < nchunks) ? xraw : 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[rb][e] = fmaf(xv, af[e], acc[rb][e]);
          }
        }
      }
    }
    // Lane l holds partial sums of the columns (l % LPR) * 8 .. + 7.  They are summed over each row
    // of sixteen lanes inside the vector ALU; the first LPR lanes of every row leave the row's sums
    // in LDS, and the exchange wave adds the sixteen rows of the workgroup in a fixed order.
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      if (RB == 1 || rb < nrows) {
        float d[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) d[e] = row_sum_same_group<LPR>(acc[rb][e]);
        if ((lane & 15) < LPR) {
          float* dst = &red[wave * 4 + (lane >> 4)][rb][(lane & 15) * 8];
          *reinterpret_cast<float4*>(dst) = make_float4(d[0], d[1], d[2], d[3]);
          *reinterpret_cast<float4*>(dst + 4) = make_float4(d[4], d[5], d[6], d[7]);
        }
      }
    }
    SGMV_TRACE_POINT(3);
    lds_barrier();  // (c) red filled
  };

  shrink_block(lo, std::true_type{});
  for (int row0 = lo + RB; row0 < hi; row0 += RB) shrink_block(row0, std::false_type{});

  // One row block of the expand phase.
  auto expand_block = [&](int row0, auto first_tag) {
    constexpr bool first = decltype(first_tag)::value;
    const int nrows = min(RB, hi - row0);
    if (!first) lds_barrier();  // (d) vs / ex free
    const __amdgpu_buffer_rsrc_t rY = make_buffer(
        y + (long long)row0 * h_out + col_lo,
        ncols > 0 ? (uint32_t)((long long)(nrows - 1) * h_out + ncols) * 2u : 0u);
    lds_barrier();  // (e) vs filled
    const bool complete = vs_complete != 0;
    for (int pass = 0; pass < npass; ++pass) {
      const int c = pass * CPW + cc;  // 8-column chunk within the slice
      const bool active = c * 8 < ncols;
      if (!first || pass != 0) {
        if (npass > 1) {
#pragma unroll
          for (int j = 0; j < JL; ++j)
            b[j] = buffer_load128(rB, active ? b_row0 + (uint32_t)j * row_bytes_out + (uint32_t)c * 16u : kOutOfRange);
        }
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
          yq[rb] = buffer_load128(rY, (cg == 0 && active && rb < nrows) ? (uint32_t)rb * row_bytes_out + (uint32_t)c * 16u : kOutOfRange);
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
          if (RB == 1 || rb < nrows) {
            const float vj = vs[rb][cg * JL + j];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[rb][e] = fmaf(vj, bf[e], acc[rb][e]);
          }
        }
      }
      if (INTRA) {
        // both lanes of a pair end with the pair's sum
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[rb][e] += neighbour_lane(acc[rb][e]);
      } else if (G > 1) {
        if (pass != 0) lds_barrier();  // (f) ex free
        if (cg > 0) {
#pragma unroll
          for (int rb = 0; rb < RB; ++rb) {
            if (RB == 1 || rb < nrows) {
              float* dst = &ex[(((cg - 1) * RB + rb) * CPW + cc) * 8];
              *reinterpret_cast<float4*>(dst) = make_float4(acc[rb][0], acc[rb][1], acc[rb][2], acc[rb][3]);
              *reinterpret_cast<float4*>(dst + 4) = make_float4(acc[rb][4], acc[rb][5], acc[rb][6], acc[rb][7]);
            }
          }
        }
        lds_barrier();  // (g) ex filled
        if (cg == 0) {
#pragma unroll
          for (int g = 1; g < G; ++g) {
#pragma unroll
            for (int rb = 0; rb < RB; ++rb) {
              if (RB == 1 || rb < nrows) {
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
      if (cg == 0) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
          float yf[8];
          unpack8<DT>(yq[rb], yf);
          uint4 out;
          out.x = pack2<DT>(yf[0] + scale * acc[rb][0], yf[1] + scale * acc[rb][1]);
          out.y = pack2<DT>(yf[2] + scale * acc[rb][2], yf[3] + scale * acc[rb][3]);
          out.z = pack2<DT>(yf[4] + scale * acc[rb][4], yf[5] + scale * acc[rb][5]);
          out.w = pack2<DT>(yf[6] + scale * acc[rb][6], yf[7] + scale * acc[rb][7]);
          buffer_store128(rY, (active && rb < nrows && complete) ? (uint32_t)rb * row_bytes_out + (uint32_t)c * 16u : kOutOfRange, out);
        }
      }
    }
  };

  expand_block(lo, std::true_type{});
  for (int row0 = lo + RB; row0 < hi; row0 += RB) expand_block(row0, std::false_type{});
  SGMV_TRACE_POINT(6);
  SGMV_TRACE_FLUSH(tid == 0, 0, 3);
  SGMV_TRACE_FLUSH(tid == 0, 6, 6);
  SGMV_TRACE_FLUSH(tid == 0, 8, 8);
}

// One add-on per launch.
template <class DT, int R, int G, int RB, bool BY_ROW>
__global__ __launch_bounds__(320) void add_lora_fused_kernel(
    // the first sixteen dwords are preloaded into SGPRs at wave launch: keep what the
    // first dependent loads need at the front
    const int32_t* __restrict__ seg_starts, const uint16_t* const* __restrict__ A_ptrs,
    const uint16_t* const* __restrict__ B_ptrs, const uint16_t* __restrict__ x,
    uint16_t* __restrict__ y, int kslice, int cslice, int h_in, int h_out, int n_tokens, int S,
    long long offA, long long offB, unsigned long long* exch, unsigned long long* header,
    float scale, int spin_limit, int n_segs) {
  // grid (fused_grid_x, S, rows): blockIdx.x is the fastest-varying part of the linear id by
  // which workgroups are dealt to the XCDs, so the S workgroups of a segment share an XCD
  // BY_ROW: the items of the grid are the rows of the batch instead of its segments, and an XCD
  // (blockIdx.x) takes a run of consecutive rows, so that rows of one segment find its weights
  // in their XCD's L2 (dealt round the XCDs, eight-row segments were read by all eight of them:
  // 16 segments of 8 rows 8.8 us)
  const int seg = BY_ROW ? blockIdx.x * gridDim.z + blockIdx.z : blockIdx.z * gridDim.x + blockIdx.x;
  if (seg >= (BY_ROW ? n_tokens : n_segs)) {  // the grid is padded to whole rows of segments
    if (threadIdx.x < 64) leave_launch_idle(header, (int)(gridDim.x * gridDim.y * gridDim.z), (int)threadIdx.x);
    return;
  }
  add_lora_fused_body<DT, R, G, RB, BY_ROW>(seg_starts, A_ptrs, B_ptrs, x, y, kslice, cslice, h_in, h_out,
                                            n_tokens, S, offA, offB, exch, header, scale, spin_limit, seg,
                                            (int)blockIdx.y, n_segs);
}

// Several independent add-ons of one shape per launch, side by side: blockIdx.z selects
// the projection's x, y and pointer arrays; each projection exchanges through its own
// stretch of the workspace.  Used while all workgroups of the launch are resident together
// (small batches); larger launches take the pipelined kernel in fused_multi_kernel.hip.
template <class DT, int R, int G, bool BY_ROW>
__global__ __launch_bounds__(320) void add_lora_fused_side_kernel(
    const int32_t* __restrict__ seg_starts, int kslice, int cslice, int h_in, int h_out, int n_tokens,
    int S, long long offA, long long offB, unsigned long long* exch, unsigned long long* header,
    float scale, int spin_limit, int n_segs, int n_proj, FusedTable tab) {
  // grid (segments of a row, S, rows of segments x projections), as for the single add-on
  const int row = __builtin_amdgcn_readfirstlane((int)(((float)blockIdx.z + 0.5f) / (float)n_proj));
  const int z = (int)blockIdx.z - row * n_proj;
  // BY_ROW: items are rows of the batch, an XCD (blockIdx.x) taking a run of consecutive rows
  const int seg = BY_ROW ? blockIdx.x * ((int)gridDim.z / n_proj) + row : row * gridDim.x + blockIdx.x;
  if (seg >= (BY_ROW ? n_tokens : n_segs)) {  // the grid is padded to whole rows of segments
    if (threadIdx.x < 64) leave_launch_idle(header, (int)(gridDim.x * gridDim.y * gridDim.z), (int)threadIdx.x);
    return;
  }
  add_lora_fused_body<DT, R, G, 1, BY_ROW>(
      seg_starts, reinterpret_cast<const uint16_t* const*>(tab.A_ptrs[z]),
      reinterpret_cast<const uint16_t* const*>(tab.B_ptrs[z]),
      reinterpret_cast<const uint16_t*>(tab.x[z]), reinterpret_cast<uint16_t*>(tab.y[z]), kslice, cslice,
      h_in, h_out, n_tokens, S, offA, offB, exch + (long long)z * S * n_tokens * R, header, scale,
      spin_limit, seg, (int)blockIdx.y, n_segs);
}

// Workspace initialisation: zero everything, then start the generation at one so that the
// zeroed exchange words (tag 0) never match.
__global__ __launch_bounds__(256) void workspace_init_kernel(uint32_t* p, size_t n_words,
                                                             size_t header_word) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n_words; i += stride)
    p[i] = (i >= header_word && i < header_word + kGenerationCopies) ? 1u
           : i == header_word + kGenerationCopies + 1                 ? kWorkspaceMagic
                                                                      : 0u;
}

hipError_t launch_workspace_init(void* p, size_t bytes, size_t header_offset, hipStream_t st) {
  const size_t n = bytes / 4;
  if (n == 0) return hipSuccess;
  unsigned blocks = (unsigned)((n + 255) / 256);
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(workspace_init_kernel, dim3(blocks), dim3(256), 0, st, (uint32_t*)p, n,
                     header_offset / 4);
  return hipGetLastError();
}

template <class DT, int R, int G, int RB, bool BY_ROW>
static hipError_t launch_fused_t(const FusedArgs& a, hipStream_t st) {
  const int items = BY_ROW ? a.n_tokens : a.n_segs;
  hipLaunchKernelGGL((add_lora_fused_kernel<DT, R, G, RB, BY_ROW>),
                     dim3((unsigned)fused_grid_x(items), (unsigned)a.S,
                          (unsigned)((items + fused_grid_x(items) - 1) / fused_grid_x(items))),
                     dim3(320), 0, st, a.seg_starts, (const uint16_t* const*)a.A_ptrs,
                     (const uint16_t* const*)a.B_ptrs, (const uint16_t*)a.x, (uint16_t*)a.y,
                     a.kslice, a.cslice, a.h_in, a.h_out, a.n_tokens, a.S, a.offA, a.offB, a.exch,
                     a.header, a.scale, a.spin_limit, a.n_segs);
  return hipGetLastError();
}

template <class DT, int R, int G, bool BY_ROW>
static hipError_t launch_fused_side_t(const FusedArgs& a, hipStream_t st) {
  const int items = BY_ROW ? a.n_tokens : a.n_segs;
  hipLaunchKernelGGL((add_lora_fused_side_kernel<DT, R, G, BY_ROW>),
                     dim3((unsigned)fused_grid_x(items), (unsigned)a.S,
                          (unsigned)(fused_grid_items(items) / fused_grid_x(items) * a.n_proj)),
                     dim3(320), 0, st, a.seg_starts, a.kslice, a.cslice, a.h_in, a.h_out, a.n_tokens, a.S,
                     a.offA, a.offB, a.exch, a.header, a.scale, a.spin_limit, a.n_segs, a.n_proj, a.table);
  return hipGetLastError();
}

template <class DT, int R, int G>
static hipError_t launch_fused_rb(const FusedArgs& a, hipStream_t st) {
  if (a.n_proj > 0) return a.by_rows ? launch_fused_side_t<DT, R, G, true>(a, st) : launch_fused_side_t<DT, R, G, false>(a, st);
  if (a.by_rows) return launch_fused_t<DT, R, G, 1, true>(a, st);
  return launch_fused_t<DT, R, G, 1, false>(a, st);
}

template <class DT, int R>
static hipError_t launch_fused_g(const FusedArgs& a, hipStream_t st) {
  switch (a.G) {
    case 1: if constexpr (R <= 16) return launch_fused_rb<DT, R, 1>(a, st); break;
    case 2: if constexpr (R <= 32) return launch_fused_rb<DT, R, 2>(a, st); break;
    case 4: return launch_fused_rb<DT, R, 4>(a, st);
    case 8: return launch_fused_rb<DT, R, 8>(a, st);
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
