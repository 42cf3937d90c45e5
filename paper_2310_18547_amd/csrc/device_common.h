// Device-side helpers shared by the SGMV kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace sgmv {

struct F16 {};
struct BF16 {};

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

// Two packed 16-bit values -> two fp32 values (element 0 is the low half).
template <class DT>
__device__ __forceinline__ void unpack2(uint32_t u, float& lo, float& hi);

template <>
__device__ __forceinline__ void unpack2<F16>(uint32_t u, float& lo, float& hi) {
  half2_t h = __builtin_bit_cast(half2_t, u);
  lo = (float)h.x;
  hi = (float)h.y;
}
template <>
__device__ __forceinline__ void unpack2<BF16>(uint32_t u, float& lo, float& hi) {
  lo = __uint_as_float(u << 16);
  hi = __uint_as_float(u & 0xFFFF0000u);
}

template <class DT>
__device__ __forceinline__ float decode1(uint16_t b);
template <>
__device__ __forceinline__ float decode1<F16>(uint16_t b) {
  return (float)__builtin_bit_cast(_Float16, b);
}
template <>
__device__ __forceinline__ float decode1<BF16>(uint16_t b) {
  return __uint_as_float((uint32_t)b << 16);
}

// fp32 -> 16 bit, round to nearest even.
template <class DT>
__device__ __forceinline__ uint32_t encode1(float f);
template <>
__device__ __forceinline__ uint32_t encode1<F16>(float f) {
  return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
}
template <>
__device__ __forceinline__ uint32_t encode1<BF16>(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;  // keep NaN a NaN
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
template <class DT>
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  return encode1<DT>(lo) | (encode1<DT>(hi) << 16);
}

// Eight packed 16-bit values (one 128-bit load) -> eight fp32 values.
template <class DT>
__device__ __forceinline__ void unpack8(const uint4& q, float (&f)[8]) {
  unpack2<DT>(q.x, f[0], f[1]);
  unpack2<DT>(q.y, f[2], f[3]);
  unpack2<DT>(q.z, f[4], f[5]);
  unpack2<DT>(q.w, f[6], f[7]);
}

__device__ __forceinline__ uint4 load128(const void* p) {
  return *reinterpret_cast<const uint4*>(p);
}
// Streaming variant for data that is read exactly once (adapter weights).
__device__ __forceinline__ uint4 load128_stream(const void* p) {
  const uint32_t* q = reinterpret_cast<const uint32_t*>(p);
  typedef uint32_t u4 __attribute__((ext_vector_type(4)));
  u4 v = __builtin_nontemporal_load(reinterpret_cast<const u4*>(q));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store128(void* p, const uint4& v) {
  *reinterpret_cast<uint4*>(p) = v;
}

// Sum eight per-lane accumulators over all lanes that hold the same rank
// columns.  Lane l of a wave works on column group (l % LPR); lanes that differ
// in the bits above log2(LPR) hold partial sums of the same eight columns.
// Three exchange steps halve the number of live values per lane (8 -> 4 -> 2
// -> 1) while doubling the span each value covers; plain butterflies finish.
// On return every lane holds the complete sum of column
//   (l % LPR) * 8 + e_out.
template <int LPR>
__device__ __forceinline__ float reduce_lanes8(const float (&a)[8], int lane, int& e_out) {
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

// Sum of v over the lanes of the same row of sixteen lanes that have the same (lane % LPR),
// left in every such lane: data-parallel-primitive moves inside the vector ALU only (quad
// permutations for the strides 1 and 2, row rotations for 4 and 8), no trip through the LDS
// crossbar.  LPR is 1, 2, 4 or 8.
template <int LPR>
__device__ __forceinline__ float row_sum_same_group(float v) {
  auto moved = [](float f, auto ctrl) {
    const int i = __float_as_int(f);
    return __int_as_float(__builtin_amdgcn_update_dpp(i, i, decltype(ctrl)::value, 0xF, 0xF, true));
  };
  if (LPR <= 1) v += moved(v, std::integral_constant<int, 0xB1>{});   // quad_perm 1,0,3,2
  if (LPR <= 2) v += moved(v, std::integral_constant<int, 0x4E>{});   // quad_perm 2,3,0,1
  if (LPR <= 4) v += moved(v, std::integral_constant<int, 0x124>{});  // row_ror 4
  v += moved(v, std::integral_constant<int, 0x128>{});                // row_ror 8
  return v;
}

// The value the neighbouring lane (lane ^ 1) holds, by a data-parallel-primitive move inside
// the vector ALU (a quad permutation): no trip through the LDS crossbar and its latency.
__device__ __forceinline__ float neighbour_lane(float v) {
  const int i = __float_as_int(v);
  return __int_as_float(__builtin_amdgcn_update_dpp(i, i, 0xB1 /* quad_perm 1,0,3,2 */, 0xF, 0xF, true));
}

}  // namespace sgmv

// ---------------------------------------------------------------------------
// Buffer addressing.  A buffer resource carries a wave-uniform base and a byte
// length; the hardware range-checks every lane, returns zero for loads beyond
// the length and drops such stores.  Lanes are predicated by giving them the
// offset kOutOfRange, so guarded 128-bit accesses need no branches and the
// compiler can issue all of a lane's loads back to back.
namespace sgmv {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr uint32_t kOutOfRange = 0x80000000u;
constexpr int kBufferWord3 = 0x00020000;  // raw buffer, 32-bit data format

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_buffer(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, kBufferWord3);
}
template <int AUX = 0>
__device__ __forceinline__ uint4 buffer_load128(__amdgpu_buffer_rsrc_t rsrc, uint32_t byte_off) {
  u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)byte_off, 0, AUX);
  return make_uint4(v.x, v.y, v.z, v.w);
}
// The same with a wave-uniform byte offset added to the lane's (kept in a scalar register, so
// that many loads of one lane share a single offset register).
__device__ __forceinline__ uint4 buffer_load128_at(__amdgpu_buffer_rsrc_t rsrc, uint32_t lane_byte_off,
                                                   uint32_t uniform_byte_off) {
  u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)lane_byte_off, (int)uniform_byte_off, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint2 buffer_load64(__amdgpu_buffer_rsrc_t rsrc, uint32_t byte_off) {
  u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rsrc, (int)byte_off, 0, 0);
  return make_uint2(v.x, v.y);
}
// 64-bit accesses with a wave-uniform byte offset added to the lane's
__device__ __forceinline__ uint2 buffer_load64_at(__amdgpu_buffer_rsrc_t rsrc, uint32_t lane_byte_off,
                                                  uint32_t uniform_byte_off) {
  u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rsrc, (int)lane_byte_off, (int)uniform_byte_off, 0);
  return make_uint2(v.x, v.y);
}
__device__ __forceinline__ void buffer_store64_at(__amdgpu_buffer_rsrc_t rsrc, uint32_t lane_byte_off,
                                                  uint32_t uniform_byte_off, const uint2& q) {
  u32x2 v = {q.x, q.y};
  __builtin_amdgcn_raw_buffer_store_b64(v, rsrc, (int)lane_byte_off, (int)uniform_byte_off, 0);
}
__device__ __forceinline__ void buffer_store64(__amdgpu_buffer_rsrc_t rsrc, uint32_t byte_off,
                                               const uint2& q) {
  u32x2 v = {q.x, q.y};
  __builtin_amdgcn_raw_buffer_store_b64(v, rsrc, (int)byte_off, 0, 0);
}
__device__ __forceinline__ void buffer_store128(__amdgpu_buffer_rsrc_t rsrc, uint32_t byte_off,
                                                const uint4& q) {
  u32x4 v = {q.x, q.y, q.z, q.w};
  __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, (int)byte_off, 0, 0);
}

// Per-row launches: the segment that holds row `row`, i.e. the number of segment ends at or
// before it (empty segments count themselves out); n_segs when the row lies behind the last end.
// Every lane of the calling wave looks at one end per round, the loads of a round in flight
// together; the result is wave-uniform.  seg_starts has n_segs + 1 non-decreasing entries.
__device__ __forceinline__ int segment_of_row(const int32_t* __restrict__ seg_starts, int n_segs, int row, int lane) {
  int found = 0;
  for (int base = 0; base < n_segs; base += 64) {
    const int i = base + lane;
    const int end = i < n_segs ? seg_starts[i + 1] : 0x7fffffff;
    found += __popcll(__ballot(end <= row));
  }
  return __builtin_amdgcn_readfirstlane(found);
}

// Workgroup barrier that orders LDS traffic only: outstanding global loads stay
// outstanding.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

}  // namespace sgmv
