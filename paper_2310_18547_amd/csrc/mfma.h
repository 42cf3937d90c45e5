// Matrix-core helpers shared by the MFMA kernels (gfx950).
//
// v_mfma_f32_16x16x32_{f16,bf16}: lane l of a wave holds row (l % 16),
// k = 8 (l / 16) .. +7 of the first operand and column (l % 16), same k, of the
// second; it receives D[4 (l / 16) + i][l % 16], i = 0..3.
#pragma once
#include "device_common.h"

namespace sgmv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <class DT>
__device__ __forceinline__ f32x4 mfma16x16x32(const uint4& a, const uint4& b, f32x4 c);
template <>
__device__ __forceinline__ f32x4 mfma16x16x32<F16>(const uint4& a, const uint4& b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
template <>
__device__ __forceinline__ f32x4 mfma16x16x32<BF16>(const uint4& a, const uint4& b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// Split an fp32 value into two 16-bit parts whose sum carries ~16-22 significant bits.
template <class DT>
__device__ __forceinline__ void split16(float v, uint32_t& hi, uint32_t& lo) {
  hi = encode1<DT>(v);
  lo = encode1<DT>(v - decode1<DT>((uint16_t)hi));
}

}  // namespace sgmv
