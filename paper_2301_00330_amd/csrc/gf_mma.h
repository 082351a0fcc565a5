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
// bf16, 32 x 32 x 16 (v_mfma_f32_32x32x16_bf16): A: lane holds row lane % 32, k = 8 * (lane / 32) .. + 7;
// B alike with the column; D: element v of the lane is row 8 * (v / 4) + 4 * (lane / 32) + v % 4 of
// column lane % 32.  A register-only loop of it measures 2.47 PFLOP/s on MI355X, one of the
// 16 x 16 x 32 form 1.40 PFLOP/s, so MFMA-bound bf16 loops use this one.
typedef float f32x16 __attribute__((ext_vector_type(16)));
__device__ __forceinline__ f32x16 mma32(const uint4& a, const uint4& b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                 0, 0, 0);
}
__device__ __forceinline__ f32x4 mma16(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}


// 16 bytes at the natural alignment of one element
template <class T> struct Unal;
template <> struct __attribute__((packed, aligned(2))) Unal<bf16_t> { uint32_t w[4]; };
template <> struct __attribute__((packed, aligned(4))) Unal<float> { uint32_t w[4]; };

// 16 bytes from an element-aligned address.  Loads near the ends of a tensor are issued at an
// offset clamped into the tensor; realign() then shifts the vector by the difference, and the
// elements whose own address lies outside the tensor come out as zeros.
template <class T>
__device__ __forceinline__ uint4 load_vec(const T* p) {
  const Unal<T> v = *reinterpret_cast<const Unal<T>*>(p);
  return make_uint4(v.w[0], v.w[1], v.w[2], v.w[3]);
}

template <class T>
__device__ __forceinline__ uint4 realign(const uint4& v, int sh) {  // out[e] = in[e + sh]
  constexpr int VE = Mma<T>::VE;
  if (sh == 0) return v;
  if (sh >= VE || sh <= -VE) return make_uint4(0, 0, 0, 0);
  uint64_t lo = (uint64_t)v.x | ((uint64_t)v.y << 32), hi = (uint64_t)v.z | ((uint64_t)v.w << 32);
  int bits = sh * 8 * (int)sizeof(T);  // 0 < |bits| < 128
  if (bits > 0) {
    if (bits >= 64) { lo = hi >> (bits - 64); hi = 0; }
    else { lo = (lo >> bits) | (hi << (64 - bits)); hi >>= bits; }
  } else {
    bits = -bits;
    if (bits >= 64) { hi = lo << (bits - 64); lo = 0; }
    else { hi = (hi << bits) | (lo >> (64 - bits)); lo <<= bits; }
  }
  return make_uint4((uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32));
}

}  // namespace gf
