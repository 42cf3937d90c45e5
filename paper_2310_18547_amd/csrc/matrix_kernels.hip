// MFMA path of SGMV for long (prefill-shaped) segments, gfx950.
//
// When a segment holds hundreds of rows, the per-segment product really is a
// dense contraction -- the reason the paper gives for grouping the requests of
// one adapter (section "Segmented Gather Matrix-Vector Multiplication", kernel
// schedule paragraph: higher operational intensity, matrix units) -- and at
// ranks up to 64 the vector ALUs can no longer keep up with HBM: the shrink
// needs r FLOP per byte of x and the expand r/2 FLOP per byte of y.  All
// kernels here are still bound by HBM (x is read once, y is read and written
// once); the matrix cores only have to be fast enough not to matter, so the
// code is organised around how x and y stream, not around MFMA utilisation.
//
// The kernels use v_mfma_f32_16x16x32_{f16,bf16}.  Its operands want eight
// consecutive k per lane: lane l of a wave holds row (l % 16), k = 8 (l / 16) ..
// +7 of the first operand and column (l % 16), same k, of the second; it
// receives D[4 (l / 16) + i][l % 16], i = 0..3.  x and v are k-contiguous in
// memory, the weights A_i [h_in][r] and B_i [r][h_out] are not, so weight tiles
// are transposed once per workgroup through LDS (pairs of k packed into a dword
// on the way in, so the LDS writes are conflict-free dword writes) and are then
// reused for every row tile of the workgroup.
//
//   shrink_stream_kernel   workgroup = (k-slice, row block, segment).  The slice of A_i
//           (at most 512 deep) stays in LDS for the workgroup's lifetime; each wave walks
//           its sixteen-row tiles of x as one sequence of register banks, two in flight,
//           and never meets the other waves again after the one staging barrier.  A_i^T
//           is the first operand, so a lane ends with four consecutive columns of one
//           row and the split-K partial sums leave as 128-bit stores.
//   shrink_matrix_kernel   the same partial sums for slices too deep for the LDS: the
//           slice is walked in chunks of 256 k that are restaged between barriers.
//   finalize_v_kernel      sums the split-K partial sums in ascending order and writes v
//           as a high and a low 16-bit part plus a range factor per row (binary16).
//   expand_matrix_kernel   workgroup = (strip of 256 columns, block of rows, segment);
//           v is the first operand and the strip of B_i (kept in registers) the second,
//           tile t of a wave holding columns 4 n + t, so a lane ends with four
//           consecutive columns (8 bytes) of four rows and every 64-bit access of y by
//           a wave covers four rows x 128 contiguous bytes.  v stays fp32 in the
//           workspace between the kernels; it enters the matrix cores as the two 16-bit
//           parts (two MFMAs, 16 significant bits for bfloat16, 22 for binary16).
//   expand_rowwise_kernel  the same product with the operands' homes exchanged, for rank 64
//           and for binary16: a wave owns sixteen rows of the block, keeps their v in
//           registers and reads B_i's strip from LDS as it walks the strip's columns.
#include <atomic>
#include <type_traits>

#include "device_common.h"
#include "launch.h"
#include "mfma.h"
#include "trace.h"


namespace sgmv {

constexpr int kShrinkRows = 64;    // rows per shrink workgroup (four 16-row tiles)
constexpr int kShrinkChunk = 256;  // k per LDS stage
constexpr int kExpandCols = 256;   // columns per expand workgroup (64 per wave)
constexpr int kExpandRows = 64;    // rows per expand workgroup and step (sixteen per wave in the row-wise kernel)

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
  // the wave index decides the base of the wave's x buffer: told to be wave-uniform, it
  // stays in scalar registers (a per-lane base would make every load a loop over lanes)
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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
    const int k_end = m < rows_here ? klen : 0;  // one compare per load, no branches between loads
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
        xn[ks] = buffer_load128(rX, k < k_end ? (uint32_t)(m * h_in + k) * 2u : kOutOfRange);
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

// ---------------------------------------------------------------- shrink, streaming
//
// Same split-K shape and the same partial sums as shrink_matrix_kernel, for slices of
// A_i small enough to stay in LDS for the lifetime of the workgroup
// (shrink_stream_lds_bytes): the slice is transposed once, and after the one barrier
// that follows the waves never meet again.  Each wave walks its sixteen-row tiles
// (row blocks blockIdx.y, + gridDim.y, ...) as one sequence of register banks of
// kStreamBank k-steps; two banks are in flight, one being consumed by the matrix cores
// while the other loads, across tile boundaries as well, so the x stream never drains.
constexpr int kStreamBank = 8;  // 32-deep k-steps per register bank (eight 128-bit loads per lane)

// LDS holds the slice rounded up to whole banks, the surplus zero, so that the
// matrix-core loop needs no guards.
__host__ __device__ constexpr int stream_kpad(int kslice) {
  return (kslice + 32 * kStreamBank - 1) / (32 * kStreamBank) * (32 * kStreamBank);
}
size_t shrink_stream_lds_bytes(int r, int kslice) {
  return (size_t)(stream_kpad(kslice) / 8) * ((r + 15) / 16 * 16 + 1) * 16;
}

// Waves (sixteen-row tiles) per workgroup: at rank 64 the slice of A_i is 65 KiB, so eight
// waves share it, which lets all workgroups of a prefill-sized call be resident at once.
constexpr int stream_waves(int r) { return r > 32 ? 8 : 4; }

// Sum of the split-K parts of four consecutive k of one row (ascending order), then the two
// 16-bit operand parts of the MFMA expand and the row's range factor: binary16 has a narrow
// range, so for F16 a row whose largest |v| reaches 2^14 is scaled down by an exact power of
// two and `undo` restores the fp32 result (1 otherwise).  The R / 4 lanes that hold a row are
// consecutive lanes of a wave, and every lane of the wave calls this (live or not).
template <class DT, int R>
__device__ __forceinline__ void finalize_quad(const float* __restrict__ first_part, int nparts,
                                              long long pstride, bool live, uint16_t* vh_at,
                                              uint16_t* vl_at, float* undo_at, bool row_leader) {
  constexpr int GPR = R / 4;  // lanes per row
  constexpr int PB = 16;      // parts with their loads in flight together
  float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int pb = 0; pb < nparts; pb += PB) {
    float4 q[PB];
#pragma unroll
    for (int i = 0; i < PB; ++i)
      q[i] = *reinterpret_cast<const float4*>(first_part + min(pb + i, nparts - 1) * pstride);
#pragma unroll
    for (int i = 0; i < PB; ++i) {
      if (pb + i < nparts) {
        sum.x += q[i].x; sum.y += q[i].y; sum.z += q[i].z; sum.w += q[i].w;
      }
    }
  }
  float f[4] = {sum.x, sum.y, sum.z, sum.w};
  float un = 1.f;
  if (std::is_same<DT, F16>::value) {
    float amax = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) amax = fmaxf(amax, fabsf(f[i]));
#pragma unroll
    for (int msk = 1; msk < GPR; msk <<= 1) amax = fmaxf(amax, __shfl_xor(amax, msk, 64));
    if (amax >= 16384.f && amax < 3.0e38f) {
      const int e = ((__float_as_uint(amax) >> 23) & 0xFF) - 127 - 13;  // amax * 2^-e < 2^14
      const float down = __uint_as_float((uint32_t)(127 - e) << 23);
      un = __uint_as_float((uint32_t)(127 + e) << 23);
#pragma unroll
      for (int i = 0; i < 4; ++i) f[i] *= down;
    }
  }
  uint32_t h[4], l[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) split16<DT>(f[i], h[i], l[i]);
  if (live) {
    *reinterpret_cast<uint2*>(vh_at) = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
    *reinterpret_cast<uint2*>(vl_at) = make_uint2(l[0] | (l[1] << 16), l[2] | (l[3] << 16));
    if (row_leader) *undo_at = un;
  }
}

// P add-ons that read the same x share one pass over it: P slices of A_i side by side in LDS, P
// sets of partial sums (P = 1: the plain shrink).
template <class DT, int R, int P>
__device__ __forceinline__ void shrink_stream_body(
    const uint16_t* __restrict__ x, const uint16_t* const* const (&A_ptrs)[P],
    const int32_t* __restrict__ seg_starts, float* const (&partials)[P], int h_in, int kslice,
    int n_tokens, long long layer_off, unsigned long long* header) {
  constexpr int NW = stream_waves(R);
  constexpr int NT = 64 * NW;
  constexpr int ROWS = 16 * NW;  // rows per workgroup and step
  constexpr int NTILE = (R + 15) / 16;
  constexpr int RPAD = NTILE * 16;
  constexpr int CG = R / 8;
  constexpr int BLK = RPAD + 1;  // 16-byte slots per block of 8 k: column n of A_i in slot n
  constexpr int XB = kStreamBank;
  constexpr int AB = 4;          // staging items (two 128-bit loads each) per thread and batch
  extern __shared__ __align__(16) uint32_t at[];  // (stream_kpad(kslice) / 8) * BLK slots

  const int seg = blockIdx.z, s = blockIdx.x, tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  SGMV_TRACE_DECL
  SGMV_TRACE_POINT(0);
  const int lo = seg_starts[seg], hi = seg_starts[seg + 1];
  if ((int)blockIdx.y * ROWS >= hi - lo) return;
  const uint16_t* A[P];
  bool any = false;
#pragma unroll
  for (int p = 0; p < P; ++p) {
    A[p] = A_ptrs[p][seg];
    any = any || A[p] != nullptr;
  }
  if (!any) return;
  const int k0 = s * kslice;
  const int klen = min(h_in, k0 + kslice) - k0;
  if (klen <= 0) return;
  SGMV_TRACE_POINT(8);
  const int m = lane & 15, g = lane >> 4;

  // this wave's tiles: rows lo + ROWS (blockIdx.y + j gridDim.y) + 16 wave .. +15, j = 0 .. my_tiles-1
  const int span = hi - lo - wave * 16;
  const int wave_blocks = span > 0 ? (span + ROWS - 1) / ROWS : 0;
  const int my_tiles = wave_blocks > (int)blockIdx.y
                           ? (wave_blocks - (int)blockIdx.y + (int)gridDim.y - 1) / (int)gridDim.y
                           : 0;
  const int nsteps = (klen + 31) >> 5;
  const int nb = (nsteps + XB - 1) / XB;  // banks per tile
  const int total = my_tiles * nb;        // banks of this wave
  const uint32_t x_lane = (uint32_t)(m * h_in + g * 8) * 2u;

  // bank b of tile j: k-steps XB b .. XB b + XB - 1; lane (m, g) takes row m, k = 32 step + 8 g .. +7
  auto load_bank = [&](uint4 (&q)[XB], int j, int b) {
    // a bank past the wave's last tile (j >= my_tiles) has no rows: an empty buffer, every
    // lane out of range, no memory traffic
    const int row0 = j < my_tiles ? lo + ((int)blockIdx.y + j * (int)gridDim.y) * ROWS + wave * 16 : lo;
    const int rows_here = j < my_tiles ? min(16, hi - row0) : 0;
    const __amdgpu_buffer_rsrc_t rX = make_buffer(
        x + (long long)row0 * h_in + k0,
        rows_here > 0 ? (uint32_t)((long long)(rows_here - 1) * h_in + klen) * 2u : 0u);
    const int k_end = m < rows_here ? klen - g * 8 : 0;  // rows past the segment read as zeros
#pragma unroll
    for (int i = 0; i < XB; ++i) {
      const int k = (b * XB + i) * 32;
      q[i] = buffer_load128(rX, k < k_end ? x_lane + (uint32_t)k * 2u : kOutOfRange);
    }
  };

  // ---- stage the slice of A_i, transposed; the first two banks of x follow the first
  // batch of its loads, so they are in flight while the slice is placed
  uint4 q0[XB], q1[XB];
  const int kpad = stream_kpad(kslice);
  const int slice_words = (kpad >> 3) * BLK * 4;  // LDS dwords of one add-on's slice
#pragma unroll
  for (int p = 0; p < P; ++p) {
    // an add-on without an adapter for this segment: an empty buffer, its slice reads as zeros
    const __amdgpu_buffer_rsrc_t rA = make_buffer(
        A[p] != nullptr ? A[p] + layer_off + (long long)k0 * R : x, A[p] != nullptr ? (uint32_t)klen * R * 2u : 0u);
    uint32_t* const atp = at + p * slice_words;
    const int items = (kpad >> 1) * CG;  // (pair of k, eight columns); rows past klen read as zeros
    uint4 a0[AB], a1[AB];
    for (int base = 0; base < items; base += NT * AB) {
#pragma unroll
      for (int u = 0; u < AB; ++u) {
        // item = kp * CG + cg -> rows 2 kp, 2 kp + 1, columns 8 cg .. +7
        const int item = base + u * NT + tid;
        const uint32_t o = item < items ? (uint32_t)(2 * item - item % CG) * 16u : kOutOfRange;
        a0[u] = buffer_load128(rA, o);
        a1[u] = buffer_load128(rA, item < items ? o + (uint32_t)R * 2u : kOutOfRange);
      }
      if (p == 0 && base == 0) {
        load_bank(q0, 0, 0);  // banks past the wave's tiles load nothing
        load_bank(q1, nb > 1 ? 0 : 1, nb > 1 ? 1 : 0);
      }
#pragma unroll
      for (int u = 0; u < AB; ++u) {
        const int item = base + u * NT + tid;
        if (item < items) {
          const int cg = item % CG, kp = item / CG;
          const uint32_t w0[4] = {a0[u].x, a0[u].y, a0[u].z, a0[u].w};
          const uint32_t w1[4] = {a1[u].x, a1[u].y, a1[u].z, a1[u].w};
          uint32_t* blk = &atp[(kp >> 2) * BLK * 4 + (kp & 3)];  // k block, dword of the k pair
#pragma unroll
          for (int i = 0; i < 4; ++i) {  // columns 8 cg + 2 i and + 2 i + 1, column n in slot n
            blk[(8 * cg + 2 * i) * 4] = (w0[i] & 0xFFFFu) | (w1[i] << 16);
            blk[(8 * cg + 2 * i + 1) * 4] = (w0[i] >> 16) | (w1[i] & 0xFFFF0000u);
          }
        }
      }
    }
    if (R < RPAD) {  // slots no column of A_i fills
      for (int i = tid; i < (kpad >> 3) * (RPAD - R) * 4; i += NT) {
        const int blk = i / ((RPAD - R) * 4), w = i % ((RPAD - R) * 4);
        atp[(blk * BLK + R) * 4 + w] = 0u;
      }
    }
  }
  SGMV_TRACE_POINT(1);
  // LDS-only barrier: the x loads stay in flight
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  SGMV_TRACE_POINT(2);

  // ---- stream
  f32x4 acc[P][NTILE];
  int cj = 0, cb = 0;                            // bank being consumed: tile, bank of the tile
  int lj = nb > 2 ? 0 : (nb == 2 ? 1 : 2);       // next bank to load
  int lb = nb > 2 ? 2 : 0;
  auto consume = [&](const uint4 (&q)[XB]) {
    if (cb == 0) {
#pragma unroll
      for (int p = 0; p < P; ++p)
#pragma unroll
        for (int t = 0; t < NTILE; ++t) acc[p][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int i = 0; i < XB; ++i) {
      const int step = cb * XB + i;  // steps past the slice multiply zeros
#pragma unroll
      for (int p = 0; p < P; ++p)
#pragma unroll
        for (int t = 0; t < NTILE; ++t) {
          // A_i^T first: D[column 16 t + 4 g + i][token m], four consecutive columns of a row per lane
          const uint4 bt = *reinterpret_cast<const uint4*>(&at[p * slice_words + ((step * 4 + g) * BLK + t * 16 + m) * 4]);
          acc[p][t] = mfma16x16x32<DT>(bt, q[i], acc[p][t]);
        }
    }
    if (cb == nb - 1 && cj < my_tiles) {
      // lane (m, g): row m of the tile, columns 16 t + 4 g .. + 3 of every column tile: the
      // wave's stores cover the tile's rows in runs of 64 contiguous bytes (all of it, 1 KiB
      // contiguous, at rank 16)
      const int row0 = lo + ((int)blockIdx.y + cj * (int)gridDim.y) * ROWS + wave * 16;
#pragma unroll
      for (int p = 0; p < P; ++p)
#pragma unroll
        for (int t = 0; t < NTILE; ++t) {
          const int n = t * 16 + 4 * g;
          if (n < R && row0 + m < hi) {
            float* dst = &partials[p][((long long)s * n_tokens + row0 + m) * R + n];
            *reinterpret_cast<float4*>(dst) = make_float4(acc[p][t][0], acc[p][t][1], acc[p][t][2], acc[p][t][3]);
          }
        }
    }
    if (++cb == nb) {
      cb = 0;
      ++cj;
    }
  };
  auto refill = [&](uint4 (&q)[XB]) {
    load_bank(q, lj, lb);
    if (++lb == nb) {
      lb = 0;
      ++lj;
    }
  };
  // No conditions around the loads, so that waiting for one bank leaves the other's eight
  // loads in flight: the sequence is padded to pairs with banks that load and store
  // nothing (past the wave's last tile), which cost a few matrix-core steps on zeros.
  for (int i = 0; i < total; i += 2) {
    consume(q0);
    refill(q0);
    consume(q1);
    refill(q1);
  }
  SGMV_TRACE_POINT(6);
#ifdef SGMV_TRACE
  if (header != nullptr) {
    SGMV_TRACE_FLUSH(tid == 0, 0, 2);
    SGMV_TRACE_FLUSH(tid == 0, 6, 6);
    SGMV_TRACE_FLUSH(tid == 0, 8, 8);
  }
#endif
}

template <class DT, int R>
__global__ __launch_bounds__(64 * stream_waves(R), 4) void shrink_stream_kernel(
    const uint16_t* __restrict__ x, const uint16_t* const* __restrict__ A_ptrs,
    const int32_t* __restrict__ seg_starts, float* __restrict__ partials, int h_in, int kslice,
    int n_tokens, long long layer_off, unsigned long long* header) {
  const uint16_t* const* const a[1] = {A_ptrs};
  float* const part[1] = {partials};
  shrink_stream_body<DT, R, 1>(x, a, seg_starts, part, h_in, kslice, n_tokens, layer_off, header);
}

// The shrink of up to three add-ons on the same x in one pass (q / k / v, gate / up of a prefill
// batch): x, more than nine tenths of the shrink's bytes, is read once instead of once per add-on.
struct ShrinkShared {
  const uint16_t* const* A_ptrs[kSharedShrinkMost];
  float* partials[kSharedShrinkMost];
};
template <class DT, int R, int P>
__global__ __launch_bounds__(64 * stream_waves(R), 2) void shrink_stream_shared_kernel(
    const uint16_t* __restrict__ x, const int32_t* __restrict__ seg_starts, int h_in, int kslice,
    int n_tokens, long long layer_off, ShrinkShared tab) {
  const uint16_t* const* a[P];
  float* part[P];
#pragma unroll
  for (int p = 0; p < P; ++p) {
    a[p] = tab.A_ptrs[p];
    part[p] = tab.partials[p];
  }
  const uint16_t* const* const (&ar)[P] = reinterpret_cast<const uint16_t* const* const (&)[P]>(a);
  float* const (&pr)[P] = reinterpret_cast<float* const (&)[P]>(part);
  shrink_stream_body<DT, R, P>(x, ar, seg_starts, pr, h_in, kslice, n_tokens, layer_off, nullptr);
}

// ---------------------------------------------------------------- expand

// v[row][k] = sum over the split-K parts (ascending), written out as the two 16-bit
// operands the expand kernel feeds to the matrix cores: vh, vl [n_tokens][R] 16-bit,
// undo [n_tokens] fp32 (finalize_quad).  One thread handles four consecutive k of a row;
// the kernel is one memory latency long.
template <class DT, int R>
__global__ __launch_bounds__(256) void finalize_v_kernel(
    const float* __restrict__ v_parts, int nparts, uint16_t* __restrict__ vh,
    uint16_t* __restrict__ vl, float* __restrict__ undo, int n_tokens) {
  constexpr int GPR = R / 4;  // threads per row
  const long long item = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long total = (long long)n_tokens * GPR;
  const bool live = item < total;
  const long long it = live ? item : total - 1;
  const long long e0 = it * 4;  // first element (row * R + k)
  finalize_quad<DT, R>(v_parts + e0, nparts, (long long)n_tokens * R, live, vh + e0, vl + e0,
                       undo + it / GPR, it % GPR == 0);
}

// The same for the add-ons of a shared shrink in one launch: blockIdx.y is the add-on.
struct FinalizeShared {
  const float* v_parts[kSharedShrinkMost];
  uint16_t* vh[kSharedShrinkMost];
  uint16_t* vl[kSharedShrinkMost];
  float* undo[kSharedShrinkMost];
};
template <class DT, int R>
__global__ __launch_bounds__(256) void finalize_v_shared_kernel(FinalizeShared tab, int nparts, int n_tokens) {
  constexpr int GPR = R / 4;  // threads per row
  const int z = blockIdx.y;
  const long long item = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long total = (long long)n_tokens * GPR;
  const bool live = item < total;
  const long long it = live ? item : total - 1;
  const long long e0 = it * 4;  // first element (row * R + k)
  finalize_quad<DT, R>(tab.v_parts[z] + e0, nparts, (long long)n_tokens * R, live, tab.vh[z] + e0, tab.vl[z] + e0,
                       tab.undo[z] + it / GPR, it % GPR == 0);
}

// grid = (column strips, row blocks of rows_per_wg rows, n_segs); the row-block dimension
// is walked with a stride.  vh / vl / undo come from finalize_v_kernel.
//
// The product is taken as D = v B_i with the token rows in the first operand: lane
// (n = l % 16, g = l / 16) receives D[row 4 g + i][column slot n] of every 16-column tile.
// A wave owns 64 columns as four tiles, tile t holding columns 4 n + t, so a lane ends up
// with four consecutive columns (8 bytes) of rows 4 g .. 4 g + 3, and each of its four
// 64-bit accesses of y covers four rows x 128 contiguous bytes across the wave: whole
// cache lines in both directions.  (Measured on plain read-modify-write kernels of this
// shape: 5.0 TB/s, against 3.3 TB/s for 128-bit accesses that cover sixteen rows x 64
// bytes, the layout the transposed product D = B_i^T v^T would give.)
// The strip of B_i is transposed through LDS once and kept in registers as operands.  Two
// row tiles are in flight; the first two are requested before the strip is staged.
template <class DT, int R>
__global__ __launch_bounds__(256, (R <= 32 ? 4 : 3) - (std::is_same<DT, F16>::value ? 1 : 0)) void expand_matrix_kernel(
    uint16_t* __restrict__ y, const uint16_t* __restrict__ vh, const uint16_t* __restrict__ vl,
    const float* __restrict__ undo, const uint16_t* const* __restrict__ A_ptrs,
    const uint16_t* const* __restrict__ B_ptrs, const int32_t* __restrict__ seg_starts, int h_out,
    int n_tokens, long long layer_off, float scale, int rows_per_wg, unsigned long long* header) {
  constexpr int KPAD = R < 32 ? 32 : R;  // k padded to the MFMA depth
  constexpr int KSTEPS = KPAD / 32;
  constexpr int NC = kExpandCols;        // columns per workgroup
  constexpr int NT = 256;
  constexpr int CT = 4;                  // 16-column tiles (and columns per lane) of a wave
  constexpr int KPAIRS = R / 2;
  // B_i strip, transposed, as 16-byte slots {8 consecutive k of one column}:
  // bt[k / 8][slot], NC + 1 slots per k block; column c of the strip sits in slot
  // (c % 4) * (NC / 4) + c / 4, so the sixteen lanes of an operand read (columns 4 n + t,
  // n = 0..15) read consecutive slots.
  constexpr int BLK = NC + 1;
  __shared__ __align__(16) uint32_t bt[(KPAD / 8) * BLK * 4];

  const int seg = blockIdx.z, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  SGMV_TRACE_DECL
  SGMV_TRACE_POINT(0);
  const int lo = seg_starts[seg], hi = seg_starts[seg + 1];
  if ((long long)blockIdx.y * rows_per_wg >= hi - lo) return;
  const uint16_t* B = B_ptrs[seg];
  if (B == nullptr) return;
  if (A_ptrs != nullptr && A_ptrs[seg] == nullptr) return;
  SGMV_TRACE_POINT(8);
  const int c0 = blockIdx.x * NC;
  const int ncols = min(NC, h_out - c0);
  const __amdgpu_buffer_rsrc_t rB = make_buffer(
      B + layer_off + c0, (uint32_t)((long long)(R - 1) * h_out + ncols) * 2u);

  // this lane: token rows 4 g + i of a tile (i = 0..3), columns cw .. cw + 3
  const int n = lane & 15, g = lane >> 4;
  const int cw = c0 + wave * (16 * CT) + n * CT;
  const bool c_ok = cw < h_out;

  struct Tile {  // everything one row tile reads from memory
    uint2 yq[4];
    uint4 h[KSTEPS], l[KSTEPS];
    float un[4];
  };
  // the block of rows being walked
  int rbeg = lo + (int)blockIdx.y * rows_per_wg;
  int nrows = min(hi, rbeg + rows_per_wg) - rbeg;
  __amdgpu_buffer_rsrc_t rY, rH, rL;
  auto open_block = [&]() {
    rY = make_buffer(y + (long long)rbeg * h_out, (uint32_t)((long long)nrows * h_out) * 2u);
    rH = make_buffer(vh + (long long)rbeg * R, (uint32_t)(nrows * R) * 2u);
    rL = make_buffer(vl + (long long)rbeg * R, (uint32_t)(nrows * R) * 2u);
  };
  auto fetch = [&](int r0, Tile& T) {  // rows r0 .. r0+15 relative to rbeg
    // one compare per access: rows past the block and columns past h_out read as zeros
    const int ylim = c_ok ? nrows : 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = r0 + 4 * g + i;
      T.yq[i] = buffer_load64(rY, row < ylim ? (uint32_t)(row * h_out + cw) * 2u : kOutOfRange);
    }
    const int vrow = r0 + n;  // first operand: row n of the tile, k = 32 ks + 8 g .. + 7
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      const int k = ks * 32 + g * 8;
      const uint32_t voff = vrow < (k < R ? nrows : 0) ? (uint32_t)(vrow * R + k) * 2u : kOutOfRange;
      T.h[ks] = buffer_load128(rH, voff);
      T.l[ks] = buffer_load128(rL, voff);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
      T.un[i] = std::is_same<DT, F16>::value ? undo[rbeg + min(r0 + 4 * g + i, nrows - 1)] : 1.f;
  };
  Tile t0, t1;
  open_block();
  fetch(0, t0);
  if (nrows > 16) fetch(16, t1);

  // ---- stage the strip transposed: a thread takes a pair of k and eight columns
  if (R < KPAD) {
    for (int i = tid; i < (KPAD / 8) * BLK * 4; i += NT) bt[i] = 0u;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  }
  {
    constexpr int TOTAL = KPAIRS * (NC / 8);  // (k pair, 8 columns) items
    constexpr int BATCH = TOTAL / NT >= 4 ? 4 : TOTAL / NT >= 1 ? TOTAL / NT : 1;  // items per thread with their loads in flight together
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
          for (int i = 0; i < 4; ++i) {  // columns 8 cg + 2 i and + 2 i + 1, i.e. c % 4 = 2 (i % 2) (+ 1), c / 4 = 2 cg + i / 2
            blk[((2 * (i & 1)) * (NC / 4) + 2 * cg + (i >> 1)) * 4] = (a0[i] & 0xFFFFu) | (a1[i] << 16);
            blk[((2 * (i & 1) + 1) * (NC / 4) + 2 * cg + (i >> 1)) * 4] = (a0[i] >> 16) | (a1[i] & 0xFFFF0000u);
          }
        }
      }
    }
  }
  SGMV_TRACE_POINT(1);
  // LDS-only barrier: the tile loads stay in flight
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  SGMV_TRACE_POINT(2);

  // ---- second operands: tile t, lane (n, g): column 4 n + t of the wave's 64, k block 4 ks + g
  uint4 bop[KSTEPS][CT];
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
    for (int t = 0; t < CT; ++t) {
      const int pos = t * (NC / 4) + wave * 16 + n;  // column wave * 64 + 4 n + t
      bop[ks][t] = *reinterpret_cast<const uint4*>(&bt[((ks * 4 + g) * BLK + pos) * 4]);
    }

  auto finish = [&](int r0, const Tile& T) {
    f32x4 acc[CT];
#pragma unroll
    for (int t = 0; t < CT; ++t) {
      acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KSTEPS; ++ks) {
        acc[t] = mfma16x16x32<DT>(T.l[ks], bop[ks][t], acc[t]);
        acc[t] = mfma16x16x32<DT>(T.h[ks], bop[ks][t], acc[t]);
      }
    }
    // acc[t][i] is column cw + t of row 4 g + i
    const int ylim = c_ok ? nrows : 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float yf[4];
      unpack2<DT>(T.yq[i].x, yf[0], yf[1]);
      unpack2<DT>(T.yq[i].y, yf[2], yf[3]);
      const float sc = scale * T.un[i];
      float o[4];
#pragma unroll
      for (int t = 0; t < CT; ++t) o[t] = yf[t] + sc * acc[t][i];
      const uint2 out = make_uint2(pack2<DT>(o[0], o[1]), pack2<DT>(o[2], o[3]));
      const int row = r0 + 4 * g + i;
      buffer_store64(rY, row < ylim ? (uint32_t)(row * h_out + cw) * 2u : kOutOfRange, out);
    }
  };

  for (bool first = true;; first = false) {
    if (!first) {
      open_block();
      fetch(0, t0);
      if (nrows > 16) fetch(16, t1);
    }
    // steady state without conditions around the loads: waiting for one tile leaves the
    // other tile's loads in flight
    int r = 0;
    for (; r + 48 < nrows; r += 32) {
      finish(r, t0);
      fetch(r + 32, t0);
      finish(r + 16, t1);
      fetch(r + 48, t1);
    }
    const int rem = nrows - r;  // 1..48 rows left
    finish(r, t0);
    if (rem > 32) fetch(r + 32, t0);
    if (rem > 16) finish(r + 16, t1);
    if (rem > 32) finish(r + 32, t0);
    // next block of this workgroup (only when the grid is smaller than the longest segment needs)
    const long long next = (long long)rbeg - lo + (long long)gridDim.y * rows_per_wg;
    if (next >= hi - lo) break;
    rbeg = lo + (int)next;
    nrows = min(hi, rbeg + rows_per_wg) - rbeg;
  }
  SGMV_TRACE_POINT(6);
#ifdef SGMV_TRACE
  if (header != nullptr) {
    SGMV_TRACE_FLUSH(tid == 0, 0, 2);
    SGMV_TRACE_FLUSH(tid == 0, 6, 6);
    SGMV_TRACE_FLUSH(tid == 0, 8, 8);
  }
#endif
}

// The expand for ranks above 32.  Same grid, operands, product and access pattern of y as
// expand_matrix_kernel, with the roles of the operands' homes exchanged: there a wave owns
// 64 columns, keeps their part of B_i in registers and reads v anew for every row tile, which
// at rank 64 costs 32 registers for B_i and as many bytes of v as of y per tile.  Here
// a wave owns sixteen rows of the block and walks the strip's four column groups: its v
// operands stay in registers for the whole strip (v is read once per workgroup row, not
// once per tile and wave), the strip of B_i, transposed through LDS once, is shared by
// the four waves and read from there as operands, and all sixteen 64-bit loads of the
// wave's part of y are in flight at once, requested before the strip is placed.
// Workgroups are short-lived on purpose: a launch has about twice as many as fit the chip
// at once, and the hardware hands the next one to whichever compute unit comes free.  (A
// variant whose workgroups stayed resident and walked several blocks each, the next
// block's loads requested as registers came free, measured 7-14 % slower: the blocks no
// longer spread evenly.)
template <class DT, int R>
__global__ __launch_bounds__(256, 4) void expand_rowwise_kernel(
    uint16_t* __restrict__ y, const uint16_t* __restrict__ vh, const uint16_t* __restrict__ vl,
    const float* __restrict__ undo, const uint16_t* const* __restrict__ A_ptrs,
    const uint16_t* const* __restrict__ B_ptrs, const int32_t* __restrict__ seg_starts, int h_out,
    int n_tokens, long long layer_off, float scale, unsigned long long* header) {
  constexpr int KPAD = R < 32 ? 32 : R;  // k padded to the MFMA depth
  constexpr int KSTEPS = KPAD / 32;
  constexpr int NC = kExpandCols;        // columns per workgroup
  constexpr int NT = 256;
  constexpr int CT = 4;                  // 16-column tiles (and columns per lane) of a group
  constexpr int NG = NC / (16 * CT);     // column groups of the strip
  constexpr int KPAIRS = R / 2;
  constexpr int ROWS = kExpandRows;
  // B_i strip, transposed, as 16-byte slots {8 consecutive k of one column}:
  // bt[k / 8][slot], NC + 1 slots per k block; column c of the strip sits in slot
  // (c % 4) * (NC / 4) + c / 4, so the sixteen lanes of an operand read (columns 4 n + t,
  // n = 0..15) read consecutive slots.
  constexpr int BLK = NC + 1;
  __shared__ __align__(16) uint32_t bt[(KPAD / 8) * BLK * 4];

  const int seg = blockIdx.z, tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  SGMV_TRACE_DECL
  SGMV_TRACE_POINT(0);
  const int lo = seg_starts[seg], hi = seg_starts[seg + 1];
  if ((long long)blockIdx.y * ROWS >= hi - lo) return;
  const uint16_t* B = B_ptrs[seg];
  if (B == nullptr) return;
  if (A_ptrs != nullptr && A_ptrs[seg] == nullptr) return;
  SGMV_TRACE_POINT(8);
  const int c0 = blockIdx.x * NC;
  const int ncols = min(NC, h_out - c0);
  const __amdgpu_buffer_rsrc_t rB = make_buffer(
      B + layer_off + c0, (uint32_t)((long long)(R - 1) * h_out + ncols) * 2u);

  // this lane: token rows 4 g + i of the wave's tile (i = 0..3), columns c0 + 64 j + 4 n .. + 3
  // of column group j
  const int n = lane & 15, g = lane >> 4;

  // ---- the strip's loads first (L2 hits mostly), so that placing the strip does not wait
  // for the loads of y from HBM that follow them
  constexpr int TOTAL = KPAIRS * (NC / 8);  // (k pair, 8 columns) items
  constexpr int ITEMS = (TOTAL + NT - 1) / NT;
  uint4 s0[ITEMS], s1[ITEMS];
#pragma unroll
  for (int b = 0; b < ITEMS; ++b) {
    const int item = b * NT + tid;  // consecutive lanes: consecutive 16 bytes of a row
    const int cg = item % (NC / 8), kp = item / (NC / 8);
    const bool in = item < TOTAL && cg * 8 < ncols;
    s0[b] = buffer_load128(rB, in ? (uint32_t)((2 * kp) * h_out + cg * 8) * 2u : kOutOfRange);
    s1[b] = buffer_load128(rB, in ? (uint32_t)((2 * kp + 1) * h_out + cg * 8) * 2u : kOutOfRange);
  }

  // y: lane offsets of rows 4 g + i in the wave's tile at the strip's first group; group j
  // adds 128 j bytes (a scalar operand); rows past the block and groups past h_out are
  // switched off per access
  uint32_t yoff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) yoff[i] = (uint32_t)((4 * g + i) * h_out + c0 + n * CT) * 2u;
  const int groups_ok = max(0, min(NG, (h_out - c0 - n * CT + 16 * CT - 1) / (16 * CT)));  // this lane's groups inside h_out

  // everything the wave reads for its sixteen rows of one block
  uint2 yq[NG][4];
  uint4 vhi[KSTEPS], vlo[KSTEPS];
  float un[4];
  __amdgpu_buffer_rsrc_t rY;
  int rows = 0;  // rows of the wave's tile inside the segment
  auto fetch = [&](int rbeg) {
    const int r0 = rbeg + wave * 16;
    rows = max(0, min(16, min(hi, rbeg + ROWS) - r0));
    rY = make_buffer(y + (long long)r0 * h_out, (uint32_t)(rows * h_out) * 2u);
    const __amdgpu_buffer_rsrc_t rH = make_buffer(vh + (long long)r0 * R, (uint32_t)(rows * R) * 2u);
    const __amdgpu_buffer_rsrc_t rL = make_buffer(vl + (long long)r0 * R, (uint32_t)(rows * R) * 2u);
    // first operand: row n of the tile, k = 32 ks + 8 g .. + 7; rows past the segment and k
    // past the rank read as zeros
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      const int k = ks * 32 + g * 8;
      const uint32_t voff = n < (k < R ? rows : 0) ? (uint32_t)(n * R + k) * 2u : kOutOfRange;
      vhi[ks] = buffer_load128(rH, voff);
      vlo[ks] = buffer_load128(rL, voff);
    }
#pragma unroll
    for (int j = 0; j < NG; ++j) {
      const int ylim = j < groups_ok ? rows : 0;  // one compare per access
#pragma unroll
      for (int i = 0; i < 4; ++i)
        yq[j][i] = buffer_load64_at(rY, 4 * g + i < ylim ? yoff[i] : kOutOfRange, (uint32_t)j * (16 * CT * 2));
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
      un[i] = std::is_same<DT, F16>::value && rows > 0 ? undo[r0 + min(4 * g + i, rows - 1)] : 1.f;
  };
  int rbeg = lo + (int)blockIdx.y * ROWS;
  fetch(rbeg);

  // ---- place the strip transposed: a thread takes pairs of k of eight columns
  if (R < KPAD) {
    for (int i = tid; i < (KPAD / 8) * BLK * 4; i += NT) bt[i] = 0u;
    lds_barrier();
  }
#pragma unroll
  for (int b = 0; b < ITEMS; ++b) {
    const int item = b * NT + tid;
    const int cg = item % (NC / 8), kp = item / (NC / 8);
    if (item < TOTAL) {
      const uint32_t a0[4] = {s0[b].x, s0[b].y, s0[b].z, s0[b].w};
      const uint32_t a1[4] = {s1[b].x, s1[b].y, s1[b].z, s1[b].w};
      uint32_t* blk = &bt[(kp >> 2) * BLK * 4 + (kp & 3)];  // k block, dword of the k pair
#pragma unroll
      for (int i = 0; i < 4; ++i) {  // columns 8 cg + 2 i and + 2 i + 1, i.e. c % 4 = 2 (i % 2) (+ 1), c / 4 = 2 cg + i / 2
        blk[((2 * (i & 1)) * (NC / 4) + 2 * cg + (i >> 1)) * 4] = (a0[i] & 0xFFFFu) | (a1[i] << 16);
        blk[((2 * (i & 1) + 1) * (NC / 4) + 2 * cg + (i >> 1)) * 4] = (a0[i] >> 16) | (a1[i] & 0xFFFF0000u);
      }
    }
  }
  SGMV_TRACE_POINT(1);
  lds_barrier();  // LDS only: the loads of y stay in flight
  SGMV_TRACE_POINT(2);

  for (;;) {
    // the operands are read from LDS where they are used: hoisted out of this loop (they do
    // not change from block to block) they would take 32 KPAD / 8 registers
    asm volatile("" ::: "memory");
#pragma unroll
    for (int j = 0; j < NG; ++j) {
      // second operands: column 64 j + 4 n + t of the strip, k block 4 ks + g
      auto operand = [&](int ks, int t) {
        const int pos = t * (NC / 4) + j * 16 + n;
        return *reinterpret_cast<const uint4*>(&bt[((ks * 4 + g) * BLK + pos) * 4]);
      };
      f32x4 acc[CT];
#pragma unroll
      for (int t = 0; t < CT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (KSTEPS == 1) {  // few registers: five workgroups per compute unit
#pragma unroll
        for (int t = 0; t < CT; ++t) {
          const uint4 bop = operand(0, t);
          acc[t] = mfma16x16x32<DT>(vlo[0], bop, acc[t]);
          acc[t] = mfma16x16x32<DT>(vhi[0], bop, acc[t]);
        }
      } else {  // the group's operands at once, the four tiles' sums advancing side by side
        uint4 bop[KSTEPS][CT];
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks)
#pragma unroll
          for (int t = 0; t < CT; ++t) bop[ks][t] = operand(ks, t);
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
#pragma unroll
          for (int t = 0; t < CT; ++t) acc[t] = mfma16x16x32<DT>(vlo[ks], bop[ks][t], acc[t]);
#pragma unroll
          for (int t = 0; t < CT; ++t) acc[t] = mfma16x16x32<DT>(vhi[ks], bop[ks][t], acc[t]);
        }
      }
      // acc[t][i] is column c0 + 64 j + 4 n + t of row 4 g + i
      const int ylim = j < groups_ok ? rows : 0;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float yf[4];
        unpack2<DT>(yq[j][i].x, yf[0], yf[1]);
        unpack2<DT>(yq[j][i].y, yf[2], yf[3]);
        const float sc = scale * un[i];
        float o[4];
#pragma unroll
        for (int t = 0; t < CT; ++t) o[t] = yf[t] + sc * acc[t][i];
        const uint2 out = make_uint2(pack2<DT>(o[0], o[1]), pack2<DT>(o[2], o[3]));
        buffer_store64_at(rY, 4 * g + i < ylim ? yoff[i] : kOutOfRange, (uint32_t)j * (16 * CT * 2), out);
      }
    }
    // next block of this workgroup (only when the grid is smaller than the longest segment needs)
    const long long next = (long long)rbeg - lo + (long long)gridDim.y * ROWS;
    if (next >= hi - lo) break;
    rbeg = lo + (int)next;
    fetch(rbeg);
  }
  SGMV_TRACE_POINT(6);
#ifdef SGMV_TRACE
  if (header != nullptr) {
    SGMV_TRACE_FLUSH(tid == 0, 0, 2);
    SGMV_TRACE_FLUSH(tid == 0, 6, 6);
    SGMV_TRACE_FLUSH(tid == 0, 8, 8);
  }
#endif
}

// ---------------------------------------------------------------- launchers

static unsigned row_blocks(int max_seg_len, int n_tokens, int rows_per_block) {
  const int longest = max_seg_len > 0 ? max_seg_len : n_tokens;
  int b = (longest + rows_per_block - 1) / rows_per_block;
  if (b < 1) b = 1;
  if (b > 1024) b = 1024;  // the kernels stride over row blocks
  return (unsigned)b;
}

// Largest LDS footprint of the streaming shrink (two workgroups per compute unit fit).
constexpr size_t kStreamMaxLds = 68 * 1024;

bool shrink_stream_fits(const ShrinkArgs& a) {
  return a.kslice % 32 == 0 && shrink_stream_lds_bytes(a.r, a.kslice) <= kStreamMaxLds;
}

bool shrink_shared_fits(const ShrinkArgs& a, int n_shared) {
  return n_shared >= 2 && n_shared <= kSharedShrinkMost && a.r <= 32 && shrink_stream_fits(a) &&
         n_shared * shrink_stream_lds_bytes(a.r, a.kslice) <= kStreamMaxLds;
}

template <class DT, int R, int P>
static hipError_t launch_shrink_shared_t(const ShrinkArgs& a, hipStream_t st) {
  dim3 grid((unsigned)a.ksplit, row_blocks(a.max_seg_len, a.n_tokens, 16 * stream_waves(R)), (unsigned)a.n_segs);
  auto kernel = shrink_stream_shared_kernel<DT, R, P>;
  static std::atomic<bool> enabled[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!enabled[dev].load(std::memory_order_acquire)) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)kStreamMaxLds);
    if (e != hipSuccess) return e;
    enabled[dev].store(true, std::memory_order_release);
  }
  ShrinkShared tab;
  for (int i = 0; i < kSharedShrinkMost; ++i) {
    tab.A_ptrs[i] = i < P ? (const uint16_t* const*)a.A_shared[i] : nullptr;
    tab.partials[i] = i < P ? a.partials_shared[i] : nullptr;
  }
  hipLaunchKernelGGL(kernel, grid, dim3(64 * stream_waves(R)), P * shrink_stream_lds_bytes(R, a.kslice), st,
                     (const uint16_t*)a.x, a.seg_starts, a.h_in, a.kslice, a.n_tokens, a.layer_off, tab);
  return hipGetLastError();
}

template <class DT, int R>
static hipError_t launch_shrink_shared_p(const ShrinkArgs& a, hipStream_t st) {
  switch (a.n_shared) {
    case 2: return launch_shrink_shared_t<DT, R, 2>(a, st);
    case 3: return launch_shrink_shared_t<DT, R, 3>(a, st);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_shrink_matrix_shared(const ShrinkArgs& a, hipStream_t st) {
  if (a.n_segs > 65535 || !shrink_shared_fits(a, a.n_shared)) return hipErrorInvalidValue;
  switch (a.r) {  // rank 64: eight waves per workgroup and slices of 66 KB, left to one add-on at a time
    case 8: return a.bf16 ? launch_shrink_shared_p<BF16, 8>(a, st) : launch_shrink_shared_p<F16, 8>(a, st);
    case 16: return a.bf16 ? launch_shrink_shared_p<BF16, 16>(a, st) : launch_shrink_shared_p<F16, 16>(a, st);
    case 32: return a.bf16 ? launch_shrink_shared_p<BF16, 32>(a, st) : launch_shrink_shared_p<F16, 32>(a, st);
  }
  return hipErrorInvalidValue;
}

template <class DT, int R>
static hipError_t launch_shrink_matrix_t(const ShrinkArgs& a, hipStream_t st) {
  dim3 grid((unsigned)a.ksplit, row_blocks(a.max_seg_len, a.n_tokens, kShrinkRows), (unsigned)a.n_segs);
  if (shrink_stream_fits(a)) {
    grid.y = row_blocks(a.max_seg_len, a.n_tokens, 16 * stream_waves(R));
    auto kernel = shrink_stream_kernel<DT, R>;
    // more than 64 KiB of dynamic LDS is enabled once per device (zero-initialised flags;
    // setting the attribute twice is harmless)
    static std::atomic<bool> enabled[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!enabled[dev].load(std::memory_order_acquire)) {
      const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize,
                                               (int)kStreamMaxLds);
      if (e != hipSuccess) return e;
      enabled[dev].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(kernel, grid, dim3(64 * stream_waves(R)), shrink_stream_lds_bytes(R, a.kslice), st,
                       (const uint16_t*)a.x, (const uint16_t* const*)a.A_ptrs, a.seg_starts, a.partials,
                       a.h_in, a.kslice, a.n_tokens, a.layer_off, a.header);
    return hipGetLastError();
  }
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
  // v -> 16-bit operand pairs (unless a shared launch has prepared them), then the expand proper
  if (!a.operands_ready) {
    const long long items = (long long)a.n_tokens * (R / 4);
    hipLaunchKernelGGL((finalize_v_kernel<DT, R>), dim3((unsigned)((items + 255) / 256)), dim3(256), 0,
                       st, a.v_parts, a.nparts, a.vh, a.vl, a.undo, a.n_tokens);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
  }
  // measured: with long segments the row-wise kernel is ahead at rank 64 (8-15 %) and for binary16
  // at every rank (2-3 %; the range factors cost the other one its fourth workgroup per compute
  // unit).  With segments shorter than a block only the first of its waves would have rows, and
  // the column-owning kernel, whose four waves share every row tile, is ahead (eight segments of
  // eight rows, binary16, rank 16: 6.2 against 7.6 us).
  const int longest = a.max_seg_len > 0 ? a.max_seg_len : a.n_tokens / (a.n_segs > 0 ? a.n_segs : 1);
  if ((R > 32 || std::is_same<DT, F16>::value) && longest >= kExpandRows)
    hipLaunchKernelGGL((expand_rowwise_kernel<DT, R>), grid, dim3(256), 0, st, (uint16_t*)a.y, a.vh,
                       a.vl, a.undo, (const uint16_t* const*)a.A_ptrs,
                       (const uint16_t* const*)a.B_ptrs, a.seg_starts, a.h_out, a.n_tokens,
                       a.layer_off, a.scale, a.header);
  else
    hipLaunchKernelGGL((expand_matrix_kernel<DT, R>), grid, dim3(256), 0, st, (uint16_t*)a.y, a.vh,
                       a.vl, a.undo, (const uint16_t* const*)a.A_ptrs,
                       (const uint16_t* const*)a.B_ptrs, a.seg_starts, a.h_out, a.n_tokens,
                       a.layer_off, a.scale, kExpandRows, a.header);
  return hipGetLastError();
}

template <class DT, int R>
static hipError_t launch_finalize_shared_t(const ExpandArgs* es, int n, hipStream_t st) {
  FinalizeShared tab;
  for (int i = 0; i < kSharedShrinkMost; ++i) {
    const ExpandArgs& e = es[i < n ? i : 0];
    tab.v_parts[i] = e.v_parts;
    tab.vh[i] = e.vh;
    tab.vl[i] = e.vl;
    tab.undo[i] = e.undo;
  }
  const long long items = (long long)es[0].n_tokens * (R / 4);
  hipLaunchKernelGGL((finalize_v_shared_kernel<DT, R>), dim3((unsigned)((items + 255) / 256), (unsigned)n), dim3(256), 0,
                     st, tab, es[0].nparts, es[0].n_tokens);
  return hipGetLastError();
}

// v -> operand pairs for the n add-ons of a shared shrink (their ExpandArgs with vh / vl / undo of
// their own) in one launch; their expands then run with operands_ready set.
hipError_t launch_finalize_shared(const ExpandArgs* es, int n, hipStream_t st) {
  if (n < 1 || n > kSharedShrinkMost) return hipErrorInvalidValue;
  const bool bf = es[0].bf16;
  switch (es[0].r) {
    case 8: return bf ? launch_finalize_shared_t<BF16, 8>(es, n, st) : launch_finalize_shared_t<F16, 8>(es, n, st);
    case 16: return bf ? launch_finalize_shared_t<BF16, 16>(es, n, st) : launch_finalize_shared_t<F16, 16>(es, n, st);
    case 32: return bf ? launch_finalize_shared_t<BF16, 32>(es, n, st) : launch_finalize_shared_t<F16, 32>(es, n, st);
    case 64: return bf ? launch_finalize_shared_t<BF16, 64>(es, n, st) : launch_finalize_shared_t<F16, 64>(es, n, st);
  }
  return hipErrorInvalidValue;
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
