// gfx950 matrix-core helpers: operand vector types and the two MFMA shapes used.
//
// Register layouts (lane l of a 64-wide wavefront):
//  16x16x32:  A[i = l%16][k = 8*(l/16) + j],  B[k = 8*(l/16) + j][n = l%16],  j = 0..7
//             D[i = 4*(l/16) + r][n = l%16],  r = 0..3
//  32x32x16:  A[i = l%32][k = 8*(l/32) + j],  B[k = 8*(l/32) + j][n = l%32],  j = 0..7
//             D[i = 8*(r/4) + 4*(l/32) + r%4][n = l%32],  r = 0..15
#pragma once
#include "common.hpp"

namespace wmdec {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <typename T> struct Mma;
template <> struct Mma<bf16_t> {
  __device__ static __forceinline__ f32x4 m16(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  }
  __device__ static __forceinline__ f32x16 m32(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  }
};
template <> struct Mma<f16_t> {
  __device__ static __forceinline__ f32x4 m16(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  }
  __device__ static __forceinline__ f32x16 m32(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  }
};

// two floats -> one 32-bit word holding two 16-bit values (lo = a, hi = b), round to nearest even
template <typename T> __device__ __forceinline__ uint32_t pack2(float a, float b) {
  return (uint32_t)from_float<T>(a).bits | ((uint32_t)from_float<T>(b).bits << 16);
}
// f16: built as a two-element vector so that the compiler can convert straight into the low / high half
// (v_fma_mixlo_f16 / v_fma_mixhi_f16, v_cvt_pk) instead of converting, shifting and or-ing
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
template <> __device__ __forceinline__ uint32_t pack2<f16_t>(float a, float b) {
  f16x2_t v;
  v.x = (_Float16)a;
  v.y = (_Float16)b;
  return __builtin_bit_cast(uint32_t, v);
}
// bf16 likewise: one v_cvt_pk_bf16_f32 for the pair
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
template <> __device__ __forceinline__ uint32_t pack2<bf16_t>(float a, float b) {
  bf16x2_t v;
  v.x = (__bf16)a;
  v.y = (__bf16)b;
  return __builtin_bit_cast(uint32_t, v);
}
template <typename T> __device__ __forceinline__ float unpack_lo(uint32_t w) { return to_float(T{(uint16_t)(w & 0xffffu)}); }
template <typename T> __device__ __forceinline__ float unpack_hi(uint32_t w) { return to_float(T{(uint16_t)(w >> 16)}); }

}  // namespace wmdec
