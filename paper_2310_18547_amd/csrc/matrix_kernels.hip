// MFMA path of SGMV for long (prefill-shaped) segments, gfx950.
//
// When a segment holds hundreds of rows, the per-segment product really is a
// dense contraction (the paper groups requests "to increase operational
// intensity and use Tensor Cores"), and at ranks up to 64 the vector ALUs can no
// longer keep up with HBM: the shrink needs r FLOP per byte of x and the expand
// r/2 FLOP per byte of y.  Both kernels are still bound by HBM (x is read once,
// y is read and written once); the matrix cores only have to be fast enough not
// to matter, so the code is organised around streaming x and y, not around
// MFMA utilisation.
//
// Both kernels use v_mfma_f32_16x16x32_{f16,bf16}.  Its operands want eight
// consecutive k per lane: lane l of a wave holds row (l % 16), k = 8 (l / 16) ..
// +7 of the first operand and column (l % 16), same k, of the second; it
// receives D[4 (l / 16) + i][l % 16], i = 0..3.  x and v are k-contiguous in
// memory, the weights A_i [h_in][r] and B_i [r][h_out] are not, so weight tiles
// are transposed once per workgroup through LDS (pairs of k packed into a dword
// on the way in, so the LDS writes are conflict-free dword writes) and are then
// reused for every row tile of the workgroup.
//
//   shrink  workgroup = (segment, block of 64 rows, k-slice); wave w owns rows
//           16w..16w+15 of the block.  The k-slice is walked in chunks of 256:
//           the chunk of A_i is staged transposed in LDS while the wave's x
//           loads (eight 128-bit loads per lane) are in flight.  Split-K
//           partial sums go to the workspace exactly like the vector path's.
//   expand  workgroup = (segment, strip of 256 columns, block of rows); wave w
//           owns 64 columns.  The strip of B_i is staged once and kept in
//           registers as MFMA operands.  The product is taken transposed
//           (D = B_i^T v^T) with the columns of four 16-wide tiles interleaved,
//           so that a lane ends up with 16 consecutive columns of one row and
//           y is read and written with 128-bit accesses.  v stays fp32 in the
//           workspace; it enters the matrix cores as a high and a low 16-bit
//           part (two MFMAs), which keeps ~16 significant bits.
#include <type_traits>

#include "device_common.h"
#include "launch.h"
#include "mfma.h"

namespace sgmv {

constexpr int kShrinkRows = 64;    // rows per shrink workgroup (four 16-row tiles)
constexpr int kShrinkChunk = 256;  // k per LDS stage
constexpr int kExpandCols = 256;   // columns per expand workgroup (64 per wave)
constexpr int kExpandRows = 64;    // rows per expand workgroup pass (more, smaller workgroups measured faster)
constexpr int kExpandTiles = 2;    // 16-row tiles a wave keeps in flight (deeper measured no faster)

// ---------------------------------------------------------------- shrink
//
// grid = (ksplit, row blocks, n_segs); the row-block dimension is walked with a
// stride, so any grid size is correct.  partials is [ksplit][n_tokens][R] fp32.
template <class DT, int R>
__global__ __launch_bounds__(256) void shrink_matrix_kernel(
    const uint16_t* __restrict__ x, const uint16_t* const* __restrict__ A_ptrs,
    const int32_t* __restrict__ seg_starts, float* __restrict__ partials, int h_in, int kslice,
    int n_tokens, long long layer_off) {
  constexpr int NT = 256;
  constexpr int NTILE = (R + 15) / 16;  // 16-column tiles of v
  constexpr int RPAD = NTILE * 16;
  constexpr int KC = kShrinkChunk;
  constexpr int CG = R / 8;             // 8-column groups of A_i
  constexpr int KSTEPS = KC / 32;
  // A_i chunk, transposed, as 16-byte slots {8 consecutive k of one column}:
  // at[k / 8][slot], RPAD + 1 slots per k block (the odd pitch spreads the banks).
  // Column n = 8 cg + c sits in slot c * CG + cg, so that the lanes of a staging
  // load (consecutive cg) write consecutive slots and the sixteen lanes of an
  // operand read (consecutive slots) hit distinct banks.
  constexpr int BLK = RPAD + 1;
  __shared__ __align__(16) uint32_t at[(KC / 8) * BLK * 4];

  const int seg = blockIdx.z, s = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int lo = seg_starts[seg], hi = seg_starts[seg + 1];
  if (lo >= hi) return;
  const uint16_t* A = A_ptrs[seg];
  if (A == nullptr) return;
  const int k0 = s * kslice;
  const int klen = min(h_in, k0 + kslice) - k0;
  if (klen <= 0) return;
  const __amdgpu_buffer_rsrc_t rA =
      make_buffer(A + layer_off + (long long)k0 * R, (uint32_t)klen * R * 2u);

  if (R < RPAD) {  // rows of the transposed tile that no column of A_i fills
    for (int i = tid; i < (KC / 8) * BLK * 4; i += NT) at[i] = 0u;
    __syncthreads();
  }

  const int m = lane & 15, g = lane >> 4;
  for (int rb = blockIdx.y; rb * kShrinkRows < hi - lo; rb += gridDim.y) {
    const int row0 = lo + rb * kShrinkRows + wave * 16;  // this wave's tile
    const int rows_here = max(0, min(16, hi - row0));
    // rows beyond the segment read as zeros
    const __amdgpu_buffer_rsrc_t rX = make_buffer(
        x + (long long)row0 * h_in + k0,
        rows_here > 0 ? (uint32_t)((long long)(rows_here - 1) * h_in + klen) * 2u : 0u);
    f32x4 acc[NTILE];
#pragma unroll
    for (int t = 0; t < NTILE; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Software pipeline over the k chunks: while the matrix cores work on chunk c
    // (x operands in registers, A_i chunk transposed in LDS), the loads of chunk
    // c+1 -- this wave's x operands and this thread's share of A_i -- are in flight.
    constexpr int ITEMS = (CG * (KC / 2) + NT - 1) / NT;  // (k pair, 8 columns) items per thread
    uint4 xn[KSTEPS], an0[ITEMS], an1[ITEMS];
    auto issue = [&](int kc) {
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
        const int k = kc + ks * 32 + g * 8;  // row m, k .. k+7
        xn[ks] = buffer_load128(rX, (m < rows_here && k < klen) ? (uint32_t)(m * h_in + k) * 2u : kOutOfRange);
      }
#pragma unroll
      for (int it = 0; it < ITEMS; ++it) {
        const int item = it * NT + tid;       // consecutive lanes: consecutive 16 bytes of a row
        const int cg = item % CG, kp = item / CG;
        const int k = kc + 2 * kp;
        const bool in = kp < KC / 2;           // rows past the slice read as zeros
        an0[it] = buffer_load128(rA, in ? (uint32_t)(k * R + cg * 8) * 2u : kOutOfRange);
        an1[it] = buffer_load128(rA, in ? (uint32_t)((k + 1) * R + cg * 8) * 2u : kOutOfRange);
      }
    };
    issue(0);
    for (int kc = 0; kc < klen; kc += KC) {
      uint4 xa[KSTEPS];
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) xa[ks] = xn[ks];
      __syncthreads();  // previous chunk's readers are done
      // a thread's item: a pair of k and eight columns, written transposed
#pragma unroll
      for (int it = 0; it < ITEMS; ++it) {
        const int item = it * NT + tid;
        const int cg = item % CG, kp = item / CG;
        if (kp < KC / 2) {
          const uint32_t a0[4] = {an0[it].x, an0[it].y, an0[it].z, an0[it].w};
          const uint32_t a1[4] = {an1[it].x, an1[it].y, an1[it].z, an1[it].w};
          uint32_t* blk = &at[(kp >> 2) * BLK * 4 + (kp & 3)];  // k block, dword of the k pair
#pragma unroll
          for (int i = 0; i < 4; ++i) {  // columns 8 cg + 2 i and + 2 i + 1
            blk[((2 * i) * CG + cg) * 4] = (a0[i] & 0xFFFFu) | (a1[i] << 16);
            blk[((2 * i + 1) * CG + cg) * 4] = (a0[i] >> 16) | (a1[i] & 0xFFFF0000u);
          }
        }
      }
      __syncthreads();
      if (kc + KC < klen) issue(kc + KC);
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
        if (kc + ks * 32 < klen) {
#pragma unroll
          for (int t = 0; t < NTILE; ++t) {
            const uint4 bt = *reinterpret_cast<const uint4*>(&at[((ks * 4 + g) * BLK + t * 16 + m) * 4]);
            acc[t] = mfma16x16x32<DT>(xa[ks], bt, acc[t]);
          }
        }
      }
    }
    // D[row 4g+i][slot m] of every tile; slot p holds column 8 (p % CG) + p / CG
#pragma unroll
    for (int t = 0; t < NTILE; ++t) {
      const int p = t * 16 + m;
      const int n = (p % CG) * 8 + p / CG;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int row = row0 + 4 * g + i;
        if (p < R && row < hi) partials[((long long)s * n_tokens + row) * R + n] = acc[t][i];
      }
    }
  }
}

// ---------------------------------------------------------------- expand

// v[row][k] = sum over the split-K parts (ascending), written out as the two
// 16-bit operands the expand kernel feeds to the matrix cores:
//   vh, vl  [n_tokens][R] 16-bit, undo [n_tokens] fp32.
// binary16 has a narrow range, so for F16 a row whose largest |v| reaches 2^14 is
// scaled down by an exact power of two; `undo` is the factor that restores the
// fp32 result (1 otherwise).  One thread handles eight consecutive k of a row.
template <class DT, int R>
__global__ __launch_bounds__(256) void finalize_v_kernel(
    const float* __restrict__ v_parts, int nparts, uint16_t* __restrict__ vh,
    uint16_t* __restrict__ vl, float* __restrict__ undo, int n_tokens) {
  constexpr int GPR = R / 8;  // threads per row
  const long long item = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long total = (long long)n_tokens * GPR;
  const bool live = item < total;
  const long long e0 = (live ? item : total - 1) * 8;  // first element (row * R + k)
  const long long pstride = (long long)n_tokens * R;
  float f[8];
  {
    float4 p0 = make_float4(0.f, 0.f, 0.f, 0.f), p1 = p0;
    for (int pb = 0; pb < nparts; pb += 4) {  // four parts' loads in flight together, added in order
      float4 q0[4], q1[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int p = min(pb + i, nparts - 1);
        q0[i] = *reinterpret_cast<const float4*>(v_parts + p * pstride + e0);
        q1[i] = *reinterpret_cast<const float4*>(v_parts + p * pstride + e0 + 4);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (pb + i < nparts) {
          p0.x += q0[i].x; p0.y += q0[i].y; p0.z += q0[i].z; p0.w += q0[i].w;
          p1.x += q1[i].x; p1.y += q1[i].y; p1.z += q1[i].z; p1.w += q1[i].w;
        }
      }
    }
    f[0] = p0.x; f[1] = p0.y; f[2] = p0.z; f[3] = p0.w;
    f[4] = p1.x; f[5] = p1.y; f[6] = p1.z; f[7] = p1.w;
  }
  float un = 1.f;
  if (std::is_same<DT, F16>::value) {
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(f[i]));
#pragma unroll
    for (int msk = 1; msk < GPR; msk <<= 1) amax = fmaxf(amax, __shfl_xor(amax, msk, 64));  // the row's threads
    if (amax >= 16384.f && amax < 3.0e38f) {
      const int e = ((__float_as_uint(amax) >> 23) & 0xFF) - 127 - 13;  // amax * 2^-e < 2^14
      const float down = __uint_as_float((uint32_t)(127 - e) << 23);
      un = __uint_as_float((uint32_t)(127 + e) << 23);
#pragma unroll
      for (int i = 0; i < 8; ++i) f[i] *= down;
    }
  }
  uint32_t h[8], l[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) split16<DT>(f[i], h[i], l[i]);
  if (live) {
    store128(vh + e0, make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)));
    store128(vl + e0, make_uint4(l[0] | (l[1] << 16), l[2] | (l[3] << 16), l[4] | (l[5] << 16), l[6] | (l[7] << 16)));
    if (item % GPR == 0) undo[item / GPR] = un;
  }
}

// grid = (column strips, row blocks, n_segs); the row-block dimension is walked
// with a stride.  vh / vl / undo come from finalize_v_kernel.
template <class DT, int R>
__global__ __launch_bounds__(256) void expand_matrix_kernel(
    uint16_t* __restrict__ y, const uint16_t* __restrict__ vh, const uint16_t* __restrict__ vl,
    const float* __restrict__ undo, const uint16_t* const* __restrict__ A_ptrs,
    const uint16_t* const* __restrict__ B_ptrs, const int32_t* __restrict__ seg_starts, int h_out,
    int n_tokens, long long layer_off, float scale) {
  constexpr int NT = 256;
  constexpr int KPAD = R < 32 ? 32 : R;  // k padded to the MFMA depth
  constexpr int KSTEPS = KPAD / 32;
  constexpr int NC = kExpandCols;
  constexpr int KPAIRS = R / 2;
  // B_i strip, transposed, as 16-byte slots {8 consecutive k of one column}:
  // bt[k / 8][slot], NC + 1 slots per k block; column 8 cg + c of the strip sits in
  // slot c * (NC / 8) + cg, so the lanes of a staging load write consecutive slots.
  constexpr int BLK = NC + 1;
  __shared__ __align__(16) uint32_t bt[(KPAD / 8) * BLK * 4];

  const int seg = blockIdx.z, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lo = seg_starts[seg], hi = seg_starts[seg + 1];
  if (lo >= hi) return;
  const uint16_t* B = B_ptrs[seg];
  if (B == nullptr) return;
  if (A_ptrs != nullptr && A_ptrs[seg] == nullptr) return;
  const int nblocks = (hi - lo + kExpandRows - 1) / kExpandRows;
  if ((int)blockIdx.y >= nblocks) return;
  const int c0 = blockIdx.x * NC;
  const int ncols = min(NC, h_out - c0);
  const __amdgpu_buffer_rsrc_t rB = make_buffer(
      B + layer_off + c0, (uint32_t)((long long)(R - 1) * h_out + ncols) * 2u);

  // ---- stage the strip transposed: a thread takes a pair of k and eight columns
  if (R < KPAD) {
    for (int i = tid; i < (KPAD / 8) * BLK * 4; i += NT) bt[i] = 0u;
    __syncthreads();
  }
  {
    constexpr int TOTAL = KPAIRS * (NC / 8);  // (k pair, 8 columns) items
    constexpr int BATCH = 4;                  // items per thread with their loads in flight together
    for (int base = 0; base < TOTAL; base += NT * BATCH) {
      uint4 r0[BATCH], r1[BATCH];
#pragma unroll
      for (int b = 0; b < BATCH; ++b) {
        const int item = base + b * NT + tid;  // consecutive lanes: consecutive 16 bytes of a row
        const int cg = item % (NC / 8), kp = item / (NC / 8);
        const bool in = item < TOTAL && cg * 8 < ncols;
        r0[b] = buffer_load128(rB, in ? (uint32_t)((2 * kp) * h_out + cg * 8) * 2u : kOutOfRange);
        r1[b] = buffer_load128(rB, in ? (uint32_t)((2 * kp + 1) * h_out + cg * 8) * 2u : kOutOfRange);
      }
#pragma unroll
      for (int b = 0; b < BATCH; ++b) {
        const int item = base + b * NT + tid;
        const int cg = item % (NC / 8), kp = item / (NC / 8);
        if (item < TOTAL) {
          const uint32_t a0[4] = {r0[b].x, r0[b].y, r0[b].z, r0[b].w};
          const uint32_t a1[4] = {r1[b].x, r1[b].y, r1[b].z, r1[b].w};
          uint32_t* blk = &bt[(kp >> 2) * BLK * 4 + (kp & 3)];  // k block, dword of the k pair
#pragma unroll
          for (int i = 0; i < 4; ++i) {  // columns 8 cg + 2 i and + 2 i + 1
            blk[((2 * i) * (NC / 8) + cg) * 4] = (a0[i] & 0xFFFFu) | (a1[i] << 16);
            blk[((2 * i + 1) * (NC / 8) + cg) * 4] = (a0[i] >> 16) | (a1[i] & 0xFFFF0000u);
          }
        }
      }
    }
  }
  __syncthreads();

  // ---- operands: tile t, slot (lane % 16) = 4 q + i  <->  column 32 (t / 2) + 8 q + 4 (t % 2) + i
  // of the wave's 64, so that lane group q ends up with columns 8 q .. 8 q + 7 (tiles 0, 1)
  // and 32 + 8 q .. + 7 (tiles 2, 3): each 128-bit access of the wave is a dense 64-byte run per row
  const int slot = lane & 15, g = lane >> 4;
  uint4 bop[KSTEPS][4];
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int col = wave * 64 + (t >> 1) * 32 + (slot >> 2) * 8 + (t & 1) * 4 + (slot & 3);
      const int pos = (col & 7) * (NC / 8) + (col >> 3);
      bop[ks][t] = *reinterpret_cast<const uint4*>(&bt[((ks * 4 + g) * BLK + pos) * 4]);
    }

  // this lane's output: row (lane % 16) of the tile, columns cw .. cw+7 and cw+32 .. cw+39
  const int m = lane & 15;
  const int cw = c0 + wave * 64 + g * 8;
  const bool c_ok0 = cw < h_out, c_ok1 = cw + 32 < h_out;

  struct Tile {  // everything one row tile reads from memory
    uint4 y0, y1, h[KSTEPS], l[KSTEPS];
    float un;
  };
  for (int rb = blockIdx.y; rb < nblocks; rb += gridDim.y) {
    const int rbeg = lo + rb * kExpandRows, rend = min(hi, rbeg + kExpandRows);
    const int nrows = rend - rbeg;
    const __amdgpu_buffer_rsrc_t rY = make_buffer(y + (long long)rbeg * h_out, (uint32_t)((long long)nrows * h_out) * 2u);
    const __amdgpu_buffer_rsrc_t rH = make_buffer(vh + (long long)rbeg * R, (uint32_t)(nrows * R) * 2u);
    const __amdgpu_buffer_rsrc_t rL = make_buffer(vl + (long long)rbeg * R, (uint32_t)(nrows * R) * 2u);

    auto fetch = [&](int r0, Tile& T) {  // rows r0 .. r0+15 relative to rbeg
      const int row = r0 + m;
      const bool ok = row < nrows;
      const uint32_t yoff = (uint32_t)(row * h_out + cw) * 2u;
      T.y0 = buffer_load128(rY, (ok && c_ok0) ? yoff : kOutOfRange);
      T.y1 = buffer_load128(rY, (ok && c_ok1) ? yoff + 64u : kOutOfRange);
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
        const int k = ks * 32 + g * 8;
        const uint32_t voff = (ok && k < R) ? (uint32_t)(row * R + k) * 2u : kOutOfRange;
        T.h[ks] = buffer_load128(rH, voff);
        T.l[ks] = buffer_load128(rL, voff);
      }
      T.un = std::is_same<DT, F16>::value ? undo[rbeg + min(row, nrows - 1)] : 1.f;
    };
    auto finish = [&](int r0, const Tile& T) {
      f32x4 acc[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
          acc[t] = mfma16x16x32<DT>(bop[ks][t], T.l[ks], acc[t]);
          acc[t] = mfma16x16x32<DT>(bop[ks][t], T.h[ks], acc[t]);
        }
      }
      // acc[t][i] is column cw + 32 (t / 2) + 4 (t % 2) + i of row m, i.e. element 4 t + i of {y0, y1}
      float yf[16];
      {
        float a8[8];
        unpack8<DT>(T.y0, a8);
#pragma unroll
        for (int i = 0; i < 8; ++i) yf[i] = a8[i];
        unpack8<DT>(T.y1, a8);
#pragma unroll
        for (int i = 0; i < 8; ++i) yf[8 + i] = a8[i];
      }
      const float sc = scale * T.un;
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
      const int row = r0 + m;
      const bool ok = row < nrows;
      const uint32_t yoff = (uint32_t)(row * h_out + cw) * 2u;
      buffer_store128(rY, (ok && c_ok0) ? yoff : kOutOfRange, out0);
      buffer_store128(rY, (ok && c_ok1) ? yoff + 64u : kOutOfRange, out1);
    };

    // kExpandTiles row tiles in flight: a tile's registers are refilled with the loads of the
    // tile kExpandTiles further on as soon as it is finished
    Tile tl[kExpandTiles];
#pragma unroll
    for (int i = 0; i < kExpandTiles; ++i)
      if (i * 16 < nrows) fetch(i * 16, tl[i]);
    for (int r0 = 0; r0 < nrows; r0 += 16 * kExpandTiles) {
#pragma unroll
      for (int i = 0; i < kExpandTiles; ++i) {
        const int r = r0 + 16 * i;
        if (r < nrows) {
          finish(r, tl[i]);
          if (r + 16 * kExpandTiles < nrows) fetch(r + 16 * kExpandTiles, tl[i]);
        }
      }
    }
  }
}

// ---------------------------------------------------------------- launchers

static unsigned row_blocks(int max_seg_len, int n_tokens, int rows_per_block) {
  const int longest = max_seg_len > 0 ? max_seg_len : n_tokens;
  int b = (longest + rows_per_block - 1) / rows_per_block;
  if (b < 1) b = 1;
  if (b > 1024) b = 1024;  // the kernels stride over row blocks
  return (unsigned)b;
}

template <class DT, int R>
static hipError_t launch_shrink_matrix_t(const ShrinkArgs& a, hipStream_t st) {
  dim3 grid((unsigned)a.ksplit, row_blocks(a.max_seg_len, a.n_tokens, kShrinkRows), (unsigned)a.n_segs);
  hipLaunchKernelGGL((shrink_matrix_kernel<DT, R>), grid, dim3(256), 0, st, (const uint16_t*)a.x,
                     (const uint16_t* const*)a.A_ptrs, a.seg_starts, a.partials, a.h_in, a.kslice,
                     a.n_tokens, a.layer_off);
  return hipGetLastError();
}

template <class DT>
static hipError_t launch_shrink_matrix_r(const ShrinkArgs& a, hipStream_t st) {
  switch (a.r) {
    case 8: return launch_shrink_matrix_t<DT, 8>(a, st);
    case 16: return launch_shrink_matrix_t<DT, 16>(a, st);
    case 32: return launch_shrink_matrix_t<DT, 32>(a, st);
    case 64: return launch_shrink_matrix_t<DT, 64>(a, st);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_shrink_matrix(const ShrinkArgs& a, hipStream_t st) {
  if (a.n_segs > 65535) return hipErrorInvalidValue;
  return a.bf16 ? launch_shrink_matrix_r<BF16>(a, st) : launch_shrink_matrix_r<F16>(a, st);
}

template <class DT, int R>
static hipError_t launch_expand_matrix_t(const ExpandArgs& a, hipStream_t st) {
  dim3 grid((unsigned)((a.h_out + kExpandCols - 1) / kExpandCols),
            row_blocks(a.max_seg_len, a.n_tokens, kExpandRows), (unsigned)a.n_segs);
  // v -> 16-bit operand pairs, then the expand proper
  const long long items = (long long)a.n_tokens * (R / 8);
  hipLaunchKernelGGL((finalize_v_kernel<DT, R>), dim3((unsigned)((items + 255) / 256)), dim3(256), 0,
                     st, a.v_parts, a.nparts, a.vh, a.vl, a.undo, a.n_tokens);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  hipLaunchKernelGGL((expand_matrix_kernel<DT, R>), grid, dim3(256), 0, st, (uint16_t*)a.y, a.vh,
                     a.vl, a.undo, (const uint16_t* const*)a.A_ptrs,
                     (const uint16_t* const*)a.B_ptrs, a.seg_starts, a.h_out, a.n_tokens,
                     a.layer_off, a.scale);
  return hipGetLastError();
}

template <class DT>
static hipError_t launch_expand_matrix_r(const ExpandArgs& a, hipStream_t st) {
  switch (a.r) {
    case 8: return launch_expand_matrix_t<DT, 8>(a, st);
    case 16: return launch_expand_matrix_t<DT, 16>(a, st);
    case 32: return launch_expand_matrix_t<DT, 32>(a, st);
    case 64: return launch_expand_matrix_t<DT, 64>(a, st);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_expand_matrix(const ExpandArgs& a, hipStream_t st) {
  if (a.n_segs > 65535) return hipErrorInvalidValue;
  return a.bf16 ? launch_expand_matrix_r<BF16>(a, st) : launch_expand_matrix_r<F16>(a, st);
}

}  // namespace sgmv
