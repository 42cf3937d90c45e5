// Single-launch LoRA add-on for batches whose segments hold a few rows each
// (mixed adapter popularity: some requests share an adapter, most do not), gfx950.
//
// Same idea as the single-row kernel in fused_kernel.hip -- the paper runs the
// LoRA add-on as two SGMV launches (shrink, then expand); here both share ONE
// launch, and the Split-K partial sums are handed from workgroup to workgroup per segment
// instead of through a grid synchronisation -- but a segment's rows are
// processed sixteen at a time on the matrix cores: with more than one row per
// adapter the per-segment product is a small dense contraction (the paper's
// reason for grouping requests), and the vector ALUs would spend longer on it
// than the weights take to arrive.
//
// Work split.  grid = (S, n_segs, Z).  The S workgroups (x) of a segment (y)
// each own one k-slice of A_i for the shrink and one column slice of B_i for
// the expand; blocks of sixteen rows of the segment are dealt round-robin over
// z (Z = number of row blocks of the longest segment, from the caller's hint;
// a workgroup whose z has no row block leaves at once, and a segment longer
// than the hint is still covered because every workgroup strides over row
// blocks).  A workgroup has four STREAM waves and one EXCHANGE wave:
//   * the stream waves issue all loads that depend on nothing (x, the A slice,
//     the B slice, y) at the very start through buffer resources.  The weight
//     slices are not k-contiguous in memory (A_i is [h_in][r], B_i is
//     [r][h_out]), so they are transposed once into LDS (pairs of k packed into
//     a dword on the way in) and read from there as 128-bit MFMA operands; x and
//     v are k-contiguous and go from registers / LDS straight into the matrix
//     cores.  The four waves split the k-steps of the shrink and the 64-column
//     groups of the expand.
//   * the exchange wave, which has no bulk loads in flight, adds the four
//     waves' shrink tiles, publishes them as {value, generation tag} words and
//     collects the S slices of every row (ascending order: deterministic).
// v stays fp32 in LDS and enters the expand MFMAs as a high and a low 16-bit
// part (two MFMAs, ~16-22 significant bits); for binary16 a row whose |v|
// reaches 2^14 is scaled by an exact power of two that the epilogue undoes.
// All barriers order LDS only, so outstanding global loads are never drained.
#include <atomic>
#include <type_traits>

#include "device_common.h"
#include "exchange.h"
#include "launch.h"
#include "trace.h"
#include "mfma.h"


namespace sgmv {

// LDS bytes the kernel needs for a launch shape (also used by the host to
// decide whether the shape fits).
size_t tile_lds_bytes(int r, int kslice, int cslice) {
  const int rpad = (r + 15) / 16 * 16, kpad = r < 32 ? 32 : r;
  return (size_t)(kslice / 8) * (rpad + 1) * 16 + (size_t)(kpad / 8) * (cslice + 1) * 16 +
         (size_t)2 * 4 * 16 * r * 4 + (size_t)2 * 16 * r * 4 + 2 * 16 * 4 + 16;
}

// kslice is a multiple of 32, cslice a multiple of 64 (host).
//   exch   [S][n_tokens][R] 64-bit words {fp32 value (high), tag (low)}
//   header the workspace's generation copies, then the error flag
template <class DT, int R>
__device__ __forceinline__ void tile_body(
    const int32_t* __restrict__ seg_starts, const uint16_t* const* __restrict__ A_ptrs,
    const uint16_t* const* __restrict__ B_ptrs, const uint16_t* __restrict__ x,
    uint16_t* __restrict__ y, int kslice, int cslice, int h_in, int h_out, int n_tokens, int S,
    long long offA, long long offB, unsigned long long* exch, unsigned long long* header,
    float scale, int spin_limit, const int seg) {
  constexpr int NT = 256, NW = 4;
  constexpr int CG = R / 8;              // 128-bit chunks in a row of A_i
  constexpr int NTILE = (R + 15) / 16;   // 16-column tiles of v
  constexpr int RPAD = NTILE * 16;
  constexpr int ABLK = RPAD + 1;         // 16-byte slots per block of 8 k (odd: spreads the banks)
  constexpr int KPAD = R < 32 ? 32 : R;  // the expand's k (= rank) padded to the MFMA depth
  constexpr int KSTEPS = KPAD / 32;
  constexpr int XB = 8;                  // k-steps per wave whose x operands are in flight together
  constexpr int AB = 4;                  // A staging items (two 128-bit loads each) per lane and batch
  constexpr int BB = 4;                  // B staging items per lane and batch
  constexpr int YB = 4;                  // 64-column groups per wave whose y loads are in flight together
  constexpr int EB = 4;                  // exchange elements per lane polled together
  constexpr int TILE = 16 * R;           // floats in one 16-row tile of v

  // A_i slice, transposed, as 16-byte slots {8 consecutive k of one column}:
  // at[k / 8][slot], column n = 8 cg + c in slot c * CG + cg, so the lanes of a
  // staging load (consecutive cg) write consecutive slots and the sixteen lanes of an
  // operand read (consecutive slots) hit distinct banks.  bt is the same for the
  // B_i column slice: bt[j / 8][slot], column 8 cg + c of the slice in slot c * ncg + cg.
  extern __shared__ __align__(16) uint32_t lds[];
  const int ncg = cslice >> 3;
  const int BBLK = cslice + 1;
  uint32_t* const at = lds;
  uint32_t* const bt = at + (kslice >> 3) * ABLK * 4;
  float* const red = reinterpret_cast<float*>(bt + (KPAD / 8) * BBLK * 4);  // [2][NW][TILE]
  float* const vs = red + 2 * NW * TILE;                                   // [2][TILE]
  float* const un = vs + 2 * TILE;                                         // [2][16]
  // [2] 0: a slice of the row block never arrived, its rows of y stay as they are
  int* const vs_complete = reinterpret_cast<int*>(un + 2 * 16);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  SGMV_TRACE_DECL
  SGMV_TRACE_POINT(0);
  const int s = blockIdx.x;
  const int lo = seg_starts[seg], hi = seg_starts[seg + 1];
  const uint16_t* A = A_ptrs[seg];
  const uint16_t* B = B_ptrs[seg];
  const int n_workgroups = (int)(gridDim.x * gridDim.y * gridDim.z);
  const int nrb = (hi - lo + 15) >> 4;  // row blocks of this segment
  // same decision in every workgroup that could wait for this one
  if ((int)blockIdx.z >= nrb || A == nullptr || B == nullptr) {
    if (wave == 0) leave_launch_idle(header, n_workgroups, lane);
    return;
  }
  SGMV_TRACE_POINT(8);
  const int k0 = min(h_in, s * kslice);
  const int klen = min(h_in, k0 + kslice) - k0;
  const int col_lo = min(h_out, s * cslice);
  const int ncols = min(h_out, col_lo + cslice) - col_lo;
  const int zstep = (int)gridDim.z;

  if (wave == NW) {
    // ============================================================ exchange wave
    const uint32_t tag = launch_tag(header);
    const long long stride = (long long)n_tokens * R;
    lds_barrier();  // (A) transposed A slice ready (nothing to do with it here)
    // ---- shrink phase: add the four waves' tiles, publish
    int it = 0;
    for (int rb = blockIdx.z; rb < nrb; rb += zstep, ++it) {
      const int row0 = lo + rb * 16;
      const int nel = min(16, hi - row0) * R;
      lds_barrier();  // (S) red[it & 1] filled
      const float* rd = red + (it & 1) * NW * TILE;
      unsigned long long* dst = exch + (long long)s * stride + (long long)row0 * R;
      for (int idx = lane; idx < nel; idx += 64) {
        float sum = rd[idx];
#pragma unroll
        for (int w = 1; w < NW; ++w) sum += rd[w * TILE + idx];
        const unsigned long long word = ((unsigned long long)__float_as_uint(sum) << 32) | tag;
        __hip_atomic_store(dst + idx, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    SGMV_TRACE_POINT(4);
    // ---- expand phase: collect all S slices of every row
    bool timed_out = false;
    it = 0;
    for (int rb = blockIdx.z; rb < nrb; rb += zstep, ++it) {
      const int row0 = lo + rb * 16;
      const int nel = min(16, hi - row0) * R;
      float* vd = vs + (it & 1) * TILE;
      const unsigned long long* src0 = exch + (long long)row0 * R;
      bool block_timed_out = false;
      auto collect = [&](int e0, auto eb_tag) {
        constexpr int EN = decltype(eb_tag)::value;
        float sum[EN];
#pragma unroll
        for (int e = 0; e < EN; ++e) sum[e] = 0.f;
        for (int s0 = 0; s0 < S; s0 += 8) {
          unsigned long long wv[EN][8];
          int polls = 0;
          bool ready;
          do {
#pragma unroll
            for (int e = 0; e < EN; ++e) {
              const unsigned long long* src = src0 + min(e0 + e * 64 + lane, nel - 1);
#pragma unroll
              for (int i = 0; i < 8; ++i)
                wv[e][i] = __hip_atomic_load(src + min(s0 + i, S - 1) * stride, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
            }
            ready = true;
#pragma unroll
            for (int e = 0; e < EN; ++e)
#pragma unroll
              for (int i = 0; i < 8; ++i) ready = ready && ((uint32_t)wv[e][i] == tag);
            if (!ready && ++polls >= spin_limit) {
              block_timed_out = true;
              break;
            }
          } while (!ready);
#pragma unroll
          for (int e = 0; e < EN; ++e)
#pragma unroll
            for (int i = 0; i < 8; ++i)
              sum[e] += (s0 + i < S) ? __uint_as_float((uint32_t)(wv[e][i] >> 32)) : 0.f;
        }
        // a row of v sits in R consecutive lanes of one element batch
#pragma unroll
        for (int e = 0; e < EN; ++e) {
          const int idx = e0 + e * 64 + lane;
          const bool live = idx < nel;
          float f = live ? sum[e] : 0.f;
          if (std::is_same<DT, F16>::value) {
            float amax = fabsf(f);
#pragma unroll
            for (int msk = 1; msk < R && msk < 64; msk <<= 1) amax = fmaxf(amax, __shfl_xor(amax, msk, 64));
            float restore = 1.f;
            if (amax >= 16384.f && amax < 3.0e38f) {
              const int ex = ((__float_as_uint(amax) >> 23) & 0xFF) - 127 - 13;  // amax * 2^-ex < 2^14
              f *= __uint_as_float((uint32_t)(127 - ex) << 23);
              restore = __uint_as_float((uint32_t)(127 + ex) << 23);
            }
            if (live && (idx % R) == 0) un[(it & 1) * 16 + idx / R] = restore;
          }
          if (live) vd[idx] = f;
        }
      };
      // short segments (at most 64 partial sums per slice) poll one element per lane
      if (nel <= 64) {
        collect(0, std::integral_constant<int, 1>{});
      } else {
        for (int e0 = 0; e0 < nel; e0 += 64 * EB) collect(e0, std::integral_constant<int, EB>{});
      }
      block_timed_out = __any(block_timed_out);
      timed_out = timed_out || block_timed_out;
      if (lane == 0) vs_complete[it & 1] = block_timed_out ? 0 : 1;
      SGMV_TRACE_POINT(5);
      lds_barrier();  // (E) vs[it & 1] filled
    }
    if (timed_out)
      raise_timeout(header);
    leave_launch(header, n_workgroups, tag, lane);
    SGMV_TRACE_POINT(7);
    SGMV_TRACE_FLUSH(lane == 0, 4, 7);
    return;
  }

  // ================================================================ stream waves
  const int m = lane & 15, g = lane >> 4;
  const int nsteps = (klen + 31) >> 5;    // 32-deep k-steps in this slice
  const int ngroups = (ncols + 63) >> 6;  // 64-column groups in this column slice
  const int total_a = (kslice >> 1) * CG; // (k pair, chunk) staging items of the A slice
  const int total_b = (R / 2) * ncg;      // (j pair, 8-column group) staging items of the B slice
  const uint32_t row_bytes_in = (uint32_t)h_in * 2u, row_bytes_out = (uint32_t)h_out * 2u;

  const __amdgpu_buffer_rsrc_t rA = make_buffer(A + offA + (long long)k0 * R, (uint32_t)klen * R * 2u);
  const __amdgpu_buffer_rsrc_t rB = make_buffer(
      B + offB + col_lo, ncols > 0 ? (uint32_t)((long long)(R - 1) * h_out + ncols) * 2u : 0u);

  auto x_rsrc = [&](int row0, int nrows) {
    return make_buffer(x + (long long)row0 * h_in + k0,
                       klen > 0 ? (uint32_t)((long long)(nrows - 1) * h_in + klen) * 2u : 0u);
  };
  auto y_rsrc = [&](int row0, int nrows) {
    return make_buffer(y + (long long)row0 * h_out + col_lo,
                       ncols > 0 ? (uint32_t)((long long)(nrows - 1) * h_out + ncols) * 2u : 0u);
  };
  // Offsets are kept to an add, a compare and a select per load, with no branches,
  // so that the loads below issue back to back.
  // x, k-step `step` of the slice: row m, k = 32 step + 8 g .. +7 (lanes of rows past
  // the block and k past the slice read zeros)
  const uint32_t x_lane = (uint32_t)m * row_bytes_in + (uint32_t)g * 16u;
  auto x_offset = [&](int step, int nrows) {
    const int k_end = m < nrows ? klen : 0;
    return (step * 32 + g * 8 < k_end) ? x_lane + (uint32_t)step * 64u : kOutOfRange;
  };
  // y, 64-column group `grp` of the slice: row m, columns 64 grp + 8 g .. +7 (half 0), + 32 (half 1)
  const uint32_t y_lane = (uint32_t)m * row_bytes_out + (uint32_t)g * 16u;
  auto y_offset = [&](int grp, int half, int nrows) {
    const int c_end = m < nrows ? ncols : 0;
    return (grp * 64 + g * 8 + half * 32 < c_end) ? y_lane + (uint32_t)(grp * 128 + half * 64) : kOutOfRange;
  };
  // A staging item (k pair kp, chunk cg) = kp * CG + cg: rows 2 kp and 2 kp + 1 of the
  // slice, columns 8 cg .. +7.  Items past the slice fall outside the buffer by themselves.
  auto a_offset = [&](int item) { return (uint32_t)(2 * item - (tid % CG)) * 16u; };
  // B staging item (j pair kp, 8-column group cg) = kp * ncg + cg: rows 2 kp, 2 kp + 1 of
  // B_i, columns 8 cg .. +7 of the slice.  Item -> (kp, cg) is a division by ncg, done once
  // per lane; consecutive items of a lane are NT apart and follow by increments.  Pairs past
  // the rank fall outside the buffer by themselves; column groups past a short last slice
  // read columns that are never stored.
  int b_step_kp, b_step_cg, b_kp, b_cg;
  auto b_next = [&]() {
    b_kp += b_step_kp;
    b_cg += b_step_cg;
    if (b_cg >= ncg) {
      b_cg -= ncg;
      ++b_kp;
    }
  };
  auto b_offset = [&]() { return (uint32_t)(2 * b_kp) * row_bytes_out + (uint32_t)b_cg * 16u; };

  // ---- issue everything that depends on no other workgroup: x, A, then B, y
  const int row_first = lo + (int)blockIdx.z * 16;
  const int nrows_first = min(16, hi - row_first);
  uint4 xq[XB];
  __builtin_amdgcn_sched_barrier(0);
  SGMV_TRACE_POINT(9);
  __builtin_amdgcn_sched_barrier(0);
  {
    const __amdgpu_buffer_rsrc_t rX = x_rsrc(row_first, nrows_first);
#pragma unroll
    for (int i = 0; i < XB; ++i) xq[i] = buffer_load128(rX, x_offset(wave + NW * i, nrows_first));
  }
  uint4 a0[AB], a1[AB];
#pragma unroll
  for (int b = 0; b < AB; ++b) {
    const uint32_t o = a_offset(b * NT + tid);
    a0[b] = buffer_load128(rA, o);
    a1[b] = buffer_load128(rA, o + (uint32_t)R * 2u);
  }
  __builtin_amdgcn_sched_barrier(0);  // keep x and A ahead of B and y in the memory pipe
  uint4 b0[BB], b1[BB];
  int bkp[BB], bcg[BB];
  uint4 yq[YB][2];
  auto issue_b_y = [&]() {
    const float inv_ncg = 1.0f / (float)ncg;
    // (the division sits here, behind the x and A loads, so that it does not delay them)
    b_step_kp = (int)(((float)NT + 0.5f) * inv_ncg);  // NT / ncg, wave-uniform
    b_step_cg = NT - b_step_kp * ncg;
    b_kp = (int)(((float)tid + 0.5f) * inv_ncg);      // tid / ncg, exact for these sizes
    b_cg = tid - b_kp * ncg;
#pragma unroll
    for (int b = 0; b < BB; ++b) {
      const uint32_t o = b_offset();
      bkp[b] = b_kp;
      bcg[b] = b_cg;
      b0[b] = buffer_load128(rB, o);
      b1[b] = buffer_load128(rB, o + row_bytes_out);
      b_next();
    }
    const __amdgpu_buffer_rsrc_t rY = y_rsrc(row_first, nrows_first);
#pragma unroll
    for (int gi = 0; gi < YB; ++gi) {
      yq[gi][0] = buffer_load128(rY, y_offset(wave + NW * gi, 0, nrows_first));
      yq[gi][1] = buffer_load128(rY, y_offset(wave + NW * gi, 1, nrows_first));
    }
  };
  // (issuing B and y only after the A slice is staged was measured: the partial sums are
  // published no earlier and the expand starts later)
  issue_b_y();
  __builtin_amdgcn_sched_barrier(0);
  SGMV_TRACE_POINT(1);

  // ---- slots of the transposed tiles that no load fills must read as zeros
  {
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
    if (R < RPAD) {  // columns R .. RPAD-1 of every k block of A
      for (int i = tid; i < (kslice >> 3) * (RPAD - R); i += NT)
        store128(&at[((i / (RPAD - R)) * ABLK + R + i % (RPAD - R)) * 4], zero);
    }
    if (R < KPAD) {  // k blocks R/8 .. KPAD/8-1 of B
      for (int i = tid; i < (KPAD - R) / 8 * BBLK; i += NT) store128(&bt[((R / 8) * BBLK + i) * 4], zero);
    }
  }

  // ---- stage the A slice transposed: an item is a pair of k and eight columns
  for (int base = 0; base < total_a; base += NT * AB) {
    if (base != 0) {
#pragma unroll
      for (int b = 0; b < AB; ++b) {
        const uint32_t o = a_offset(base + b * NT + tid);
        a0[b] = buffer_load128(rA, o);
        a1[b] = buffer_load128(rA, o + (uint32_t)R * 2u);
      }
    }
#pragma unroll
    for (int b = 0; b < AB; ++b) {
      const int item = base + b * NT + tid;
      const int cg = item % CG, kp = item / CG;
      if (item < total_a) {
        const uint32_t w0[4] = {a0[b].x, a0[b].y, a0[b].z, a0[b].w};
        const uint32_t w1[4] = {a1[b].x, a1[b].y, a1[b].z, a1[b].w};
        uint32_t* blk = &at[(kp >> 2) * ABLK * 4 + (kp & 3)];  // k block, dword of the k pair
#pragma unroll
        for (int i = 0; i < 4; ++i) {  // columns 8 cg + 2 i and + 2 i + 1
          blk[((2 * i) * CG + cg) * 4] = (w0[i] & 0xFFFFu) | (w1[i] << 16);
          blk[((2 * i + 1) * CG + cg) * 4] = (w0[i] >> 16) | (w1[i] & 0xFFFF0000u);
        }
      }
    }
  }
  lds_barrier();  // (A) transposed A slice ready
  SGMV_TRACE_POINT(2);

  // ---- shrink: one block of sixteen rows; the waves split the k-steps
  auto shrink_block = [&](int rb, int it, auto first_tag) {
    constexpr bool first = decltype(first_tag)::value;
    const int row0 = lo + rb * 16;
    const int nrows = min(16, hi - row0);
    const __amdgpu_buffer_rsrc_t rX = x_rsrc(row0, nrows);
    f32x4 acc[NTILE];
#pragma unroll
    for (int t = 0; t < NTILE; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int i0 = 0; i0 * NW + wave < nsteps; i0 += XB) {
      if (!first || i0 != 0) {
#pragma unroll
        for (int i = 0; i < XB; ++i) xq[i] = buffer_load128(rX, x_offset(wave + NW * (i0 + i), nrows));
      }
#pragma unroll
      for (int i = 0; i < XB; ++i) {
        const int step = wave + NW * (i0 + i);
        if (step < nsteps) {
#pragma unroll
          for (int t = 0; t < NTILE; ++t) {
            const uint4 aop = *reinterpret_cast<const uint4*>(&at[((step * 4 + g) * ABLK + t * 16 + m) * 4]);
            acc[t] = mfma16x16x32<DT>(xq[i], aop, acc[t]);
          }
        }
      }
    }
    // acc[t][i] = v[row 4g+i][slot 16t+m]; slot p holds column 8 (p % CG) + p / CG
    float* rd = red + ((it & 1) * NW + wave) * TILE;
#pragma unroll
    for (int t = 0; t < NTILE; ++t) {
      const int p = t * 16 + m;
      const int n = (p % CG) * 8 + p / CG;
      if (p < R) {
#pragma unroll
        for (int i = 0; i < 4; ++i) rd[(4 * g + i) * R + n] = acc[t][i];
      }
    }
    SGMV_TRACE_POINT(3);
    lds_barrier();  // (S) red[it & 1] filled
  };
  {
    int it = 0;
    shrink_block((int)blockIdx.z, 0, std::true_type{});
    for (int rb = (int)blockIdx.z + zstep; rb < nrb; rb += zstep) shrink_block(rb, ++it, std::false_type{});
  }

  // ---- stage the B slice transposed (while the partial sums are exchanged)
  for (int base = 0; base < total_b; base += NT * BB) {
    if (base != 0) {
#pragma unroll
      for (int b = 0; b < BB; ++b) {
        const uint32_t o = b_offset();
        bkp[b] = b_kp;
        bcg[b] = b_cg;
        b0[b] = buffer_load128(rB, o);
        b1[b] = buffer_load128(rB, o + row_bytes_out);
        b_next();
      }
    }
#pragma unroll
    for (int b = 0; b < BB; ++b) {
      const int kp = bkp[b], cg = bcg[b];
      if (kp < R / 2) {
        const uint32_t w0[4] = {b0[b].x, b0[b].y, b0[b].z, b0[b].w};
        const uint32_t w1[4] = {b1[b].x, b1[b].y, b1[b].z, b1[b].w};
        uint32_t* blk = &bt[(kp >> 2) * BBLK * 4 + (kp & 3)];  // j block, dword of the j pair
#pragma unroll
        for (int i = 0; i < 4; ++i) {  // columns 8 cg + 2 i and + 2 i + 1 of the slice
          blk[((2 * i) * ncg + cg) * 4] = (w0[i] & 0xFFFFu) | (w1[i] << 16);
          blk[((2 * i + 1) * ncg + cg) * 4] = (w0[i] >> 16) | (w1[i] & 0xFFFF0000u);
        }
      }
    }
  }

  // ---- expand: one block of sixteen rows; the waves split the 64-column groups.
  // The product is taken transposed (D = B_i^T v^T) with the columns of four 16-wide
  // tiles interleaved: tile t, slot 4 q + i <-> column 32 (t / 2) + 8 q + 4 (t % 2) + i
  // of the group, so a lane ends up with columns 8 g .. +7 and 32 + 8 g .. +7 of row m.
  auto expand_block = [&](int rb, int it, auto first_tag) {
    constexpr bool first = decltype(first_tag)::value;
    const int row0 = lo + rb * 16;
    const int nrows = min(16, hi - row0);
    const __amdgpu_buffer_rsrc_t rY = y_rsrc(row0, nrows);
    lds_barrier();  // (E) vs[it & 1] filled (and, the first time, the B slice staged)
    const int nrows_store = vs_complete[it & 1] != 0 ? nrows : 0;
    uint4 vh[KSTEPS], vl[KSTEPS];
    {
      const float* vd = vs + (it & 1) * TILE + m * R;
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
        const int k = ks * 32 + g * 8;
        uint32_t h[8], l[8];
        if (k < R) {
          const float4 p0 = *reinterpret_cast<const float4*>(vd + k);
          const float4 p1 = *reinterpret_cast<const float4*>(vd + k + 4);
          const float f[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
#pragma unroll
          for (int i = 0; i < 8; ++i) split16<DT>(f[i], h[i], l[i]);
        } else {
#pragma unroll
          for (int i = 0; i < 8; ++i) h[i] = l[i] = 0u;
        }
        vh[ks] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
        vl[ks] = make_uint4(l[0] | (l[1] << 16), l[2] | (l[3] << 16), l[4] | (l[5] << 16), l[6] | (l[7] << 16));
      }
    }
    const float sc = std::is_same<DT, F16>::value ? scale * un[(it & 1) * 16 + m] : scale;
    for (int gi0 = 0; gi0 * NW + wave < ngroups; gi0 += YB) {
      if (!first || gi0 != 0) {
#pragma unroll
        for (int gi = 0; gi < YB; ++gi) {
          yq[gi][0] = buffer_load128(rY, y_offset(wave + NW * (gi0 + gi), 0, nrows));
          yq[gi][1] = buffer_load128(rY, y_offset(wave + NW * (gi0 + gi), 1, nrows));
        }
      }
#pragma unroll
      for (int gi = 0; gi < YB; ++gi) {
        const int grp = wave + NW * (gi0 + gi);
        if (grp < ngroups) {
          f32x4 acc[4];
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
            const int col = grp * 64 + (t >> 1) * 32 + (m >> 2) * 8 + (t & 1) * 4 + (m & 3);
            const int pos = (col & 7) * ncg + (col >> 3);
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
              const uint4 bop = *reinterpret_cast<const uint4*>(&bt[((ks * 4 + g) * BBLK + pos) * 4]);
              acc[t] = mfma16x16x32<DT>(bop, vl[ks], acc[t]);
              acc[t] = mfma16x16x32<DT>(bop, vh[ks], acc[t]);
            }
          }
          // acc[t][i] is column 8 g + 32 (t / 2) + 4 (t % 2) + i of the group, row m:
          // element 4 t + i of {yq[gi][0], yq[gi][1]}
          float yf[16];
          {
            float a8[8];
            unpack8<DT>(yq[gi][0], a8);
#pragma unroll
            for (int i = 0; i < 8; ++i) yf[i] = a8[i];
            unpack8<DT>(yq[gi][1], a8);
#pragma unroll
            for (int i = 0; i < 8; ++i) yf[8 + i] = a8[i];
          }
          float o[16];
#pragma unroll
          for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) o[t * 4 + i] = yf[t * 4 + i] + sc * acc[t][i];
          uint4 out0, out1;
          out0.x = pack2<DT>(o[0], o[1]);   out0.y = pack2<DT>(o[2], o[3]);
          out0.z = pack2<DT>(o[4], o[5]);   out0.w = pack2<DT>(o[6], o[7]);
          out1.x = pack2<DT>(o[8], o[9]);   out1.y = pack2<DT>(o[10], o[11]);
          out1.z = pack2<DT>(o[12], o[13]); out1.w = pack2<DT>(o[14], o[15]);
          buffer_store128(rY, y_offset(grp, 0, nrows_store), out0);
          buffer_store128(rY, y_offset(grp, 1, nrows_store), out1);
        }
      }
    }
  };
  {
    int it = 0;
    expand_block((int)blockIdx.z, 0, std::true_type{});
    for (int rb = (int)blockIdx.z + zstep; rb < nrb; rb += zstep) expand_block(rb, ++it, std::false_type{});
  }
  SGMV_TRACE_POINT(6);
  SGMV_TRACE_FLUSH(tid == 0, 0, 3);
  SGMV_TRACE_FLUSH(tid == 0, 6, 6);
  SGMV_TRACE_FLUSH(tid == 0, 8, 9);
}

template <class DT, int R>
__global__ __launch_bounds__(320) void add_lora_tile_kernel(
    // the first sixteen dwords are preloaded into SGPRs at wave launch
    const int32_t* __restrict__ seg_starts, const uint16_t* const* __restrict__ A_ptrs,
    const uint16_t* const* __restrict__ B_ptrs, const uint16_t* __restrict__ x,
    uint16_t* __restrict__ y, int kslice, int cslice, int h_in, int h_out, int n_tokens, int S,
    long long offA, long long offB, unsigned long long* exch, unsigned long long* header,
    float scale, int spin_limit) {
  tile_body<DT, R>(seg_starts, A_ptrs, B_ptrs, x, y, kslice, cslice, h_in, h_out, n_tokens, S, offA, offB, exch,
                   header, scale, spin_limit, (int)blockIdx.y);
}

// Several add-ons of one shape side by side: blockIdx.y = add-on * n_segs + segment.  Each add-on
// has its own x, y and weight pointers (tab) and its own stretch of exchange words; the segments
// and the slicing are shared.
template <class DT, int R>
__global__ __launch_bounds__(320) void add_lora_tile_multi_kernel(
    const int32_t* __restrict__ seg_starts, int kslice, int cslice, int h_in, int h_out, int n_tokens,
    int S, long long offA, long long offB, unsigned long long* exch, unsigned long long* header,
    float scale, int spin_limit, int n_segs, FusedTable tab) {
  const int proj = (int)blockIdx.y / n_segs;
  tile_body<DT, R>(seg_starts, reinterpret_cast<const uint16_t* const*>(tab.A_ptrs[proj]),
                   reinterpret_cast<const uint16_t* const*>(tab.B_ptrs[proj]),
                   reinterpret_cast<const uint16_t*>(tab.x[proj]), reinterpret_cast<uint16_t*>(tab.y[proj]), kslice,
                   cslice, h_in, h_out, n_tokens, S, offA, offB, exch + (long long)proj * S * n_tokens * R, header,
                   scale, spin_limit, (int)blockIdx.y - proj * n_segs);
}

// LDS beyond 64 KiB per workgroup has to be enabled per kernel, once per device
static hipError_t enable_tile_lds(const void* kernel, std::atomic<bool>* enabled) {
  int dev = 0;
  hipError_t err = hipGetDevice(&dev);
  if (err != hipSuccess) return err;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!enabled[dev].load(std::memory_order_acquire)) {
    err = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kTileMaxLds);
    if (err != hipSuccess) return err;
    enabled[dev].store(true, std::memory_order_release);
  }
  return hipSuccess;
}

template <class DT, int R>
static hipError_t launch_tile_t(const TileArgs& a, hipStream_t st) {
  // A workgroup asks for more than half of the unit's LDS even when it uses less, so that no
  // two of them share a compute unit: the grid has a workgroup per segment and block of the
  // LONGEST segment, and the ones without rows, although they leave at once, hold unit slots
  // at dispatch, so that live ones were doubled up on some units while others stayed empty
  // (one long and many short segments: 10.1 us, the issue phase of every workgroup twice as long)
  const size_t lds = a.lds_bytes > kTileExclusiveLds ? a.lds_bytes : kTileExclusiveLds;
  static std::atomic<bool> enabled[2][64];  // zero-initialised; setting the attribute twice is harmless
  if (a.n_proj > 1) {
    auto kernel = add_lora_tile_multi_kernel<DT, R>;
    const hipError_t err = enable_tile_lds(reinterpret_cast<const void*>(kernel), enabled[1]);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(kernel, dim3((unsigned)a.S, (unsigned)(a.n_segs * a.n_proj), (unsigned)a.Z), dim3(320), lds,
                       st, a.seg_starts, a.kslice, a.cslice, a.h_in, a.h_out, a.n_tokens, a.S, a.offA, a.offB,
                       a.exch, a.header, a.scale, a.spin_limit, a.n_segs, a.table);
    return hipGetLastError();
  }
  auto kernel = add_lora_tile_kernel<DT, R>;
  const hipError_t err = enable_tile_lds(reinterpret_cast<const void*>(kernel), enabled[0]);
  if (err != hipSuccess) return err;
  hipLaunchKernelGGL(kernel, dim3((unsigned)a.S, (unsigned)a.n_segs, (unsigned)a.Z), dim3(320),
                     lds, st, a.seg_starts, (const uint16_t* const*)a.A_ptrs,
                     (const uint16_t* const*)a.B_ptrs, (const uint16_t*)a.x, (uint16_t*)a.y, a.kslice,
                     a.cslice, a.h_in, a.h_out, a.n_tokens, a.S, a.offA, a.offB, a.exch, a.header,
                     a.scale, a.spin_limit);
  return hipGetLastError();
}

template <class DT>
static hipError_t launch_tile_r(const TileArgs& a, hipStream_t st) {
  switch (a.r) {
    case 8: return launch_tile_t<DT, 8>(a, st);
    case 16: return launch_tile_t<DT, 16>(a, st);
    case 32: return launch_tile_t<DT, 32>(a, st);
    case 64: return launch_tile_t<DT, 64>(a, st);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_add_lora_tile(const TileArgs& a, hipStream_t st) {
  if (a.lds_bytes > kTileMaxLds || (long long)a.n_segs * (a.n_proj > 1 ? a.n_proj : 1) > 65535 || a.Z > 65535)
    return hipErrorInvalidValue;
  return a.bf16 ? launch_tile_r<BF16>(a, st) : launch_tile_r<F16>(a, st);
}

}  // namespace sgmv
