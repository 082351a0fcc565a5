// MFMA primitives shared by the GEMM-shaped kernels of libgf (gfx950).
//
// bf16: v_mfma_f32_16x16x32_bf16 -- A: lane holds row lane % 16, k = 8 * (lane / 16) .. + 7 (one
// 16-byte register quad); B: the same with the column in place of the row; D: lane holds
// rows 4 * (lane / 16) .. + 3 of column lane % 16.
// fp32: v_mfma_f32_16x16x4_f32 -- A / B: lane holds row (column) lane % 16, k = lane / 16; D as above.
#pragma once

#include "gf_internal.h"

namespace gf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <class T> struct Mma;
template <> struct Mma<bf16_t> {
  static constexpr int KSTEP = 32;  // k per MFMA
  static constexpr int BK = 64;     // k per 128-byte staged row
  static constexpr int VE = 8;      // elements per 16-byte vector
  static constexpr uint32_t FULL = 0xffu;  // element mask of a whole vector
};
template <> struct Mma<float> {
  static constexpr int KSTEP = 4;
  static constexpr int BK = 32;
  static constexpr int VE = 4;
  static constexpr uint32_t FULL = 0xfu;
};

__device__ __forceinline__ f32x4 mma16(const uint4& a, const uint4& b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mma16(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

}  // namespace gf
