// 8-bit floating point (E4M3 of the OCP 8-bit floating point specification: 1 sign bit, 4 exponent bits with
// bias 7, 3 mantissa bits, no infinities, S.1111.111 = NaN, largest magnitude 448, subnormals m * 2^-9) for the
// row-wise quantised storage of a compressed cache: conversions shared by the quantiser and the decoding step.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace meda {

constexpr float kE4M3Max = 448.0f;

// Code of a finite float with |y| <= 448: nearest representable value, ties to the even mantissa.  Integer
// arithmetic on the bit pattern, so the result does not depend on any conversion mode of the hardware.
__device__ __forceinline__ uint32_t float_to_e4m3(float y) {
  const uint32_t b = __float_as_uint(y), sign = (b >> 24) & 0x80u, a = b & 0x7fffffffu;
  uint32_t code;
  if (a < 0x3C800000u) {
    // below the smallest normal 2^-6 the grid is m * 2^-9: round |y| * 2^9 to an integer (exact product);
    // 8 is the code of 2^-6 itself
    code = (uint32_t)__float2int_rn(__uint_as_float(a) * 512.0f);
  } else {
    // keep the exponent and the top three mantissa bits, round to nearest even on the 20 bits dropped (a carry
    // runs into the exponent), then move the exponent bias from 127 to 7
    const uint32_t r = a + 0x7FFFFu + ((a >> 20) & 1u);
    code = min((r >> 20) - (120u << 3), 0x7Eu);
  }
  return sign | code;
}

// Two codes (bytes 0,1 or bytes 2,3 of `word`) as floats.
__device__ __forceinline__ void e4m3x2_to_float(uint32_t word, bool upper, float& f0, float& f1) {
#if __HIP_DEVICE_COMPILE__
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = upper ? __builtin_amdgcn_cvt_pk_f32_fp8((int)word, true)
                          : __builtin_amdgcn_cvt_pk_f32_fp8((int)word, false);
  f0 = v[0];
  f1 = v[1];
#else
  f0 = f1 = 0.f;
#endif
}

// Eight codes (8 bytes) as eight bf16 values packed in 16 bytes, element order kept.  Exact: every E4M3 value
// is a bf16 value (3 mantissa bits, exponents -9 .. 8).
__device__ __forceinline__ uint4 e4m3x8_to_bf16x8(uint2 c) {
  float f[8];
  e4m3x2_to_float(c.x, false, f[0], f[1]);
  e4m3x2_to_float(c.x, true, f[2], f[3]);
  e4m3x2_to_float(c.y, false, f[4], f[5]);
  e4m3x2_to_float(c.y, true, f[6], f[7]);
  uint4 o;
  // upper halves of two floats side by side: bytes 2,3 of the first, bytes 2,3 of the second
  o.x = __builtin_amdgcn_perm(__float_as_uint(f[1]), __float_as_uint(f[0]), 0x07060302u);
  o.y = __builtin_amdgcn_perm(__float_as_uint(f[3]), __float_as_uint(f[2]), 0x07060302u);
  o.z = __builtin_amdgcn_perm(__float_as_uint(f[5]), __float_as_uint(f[4]), 0x07060302u);
  o.w = __builtin_amdgcn_perm(__float_as_uint(f[7]), __float_as_uint(f[6]), 0x07060302u);
  return o;
}

}  // namespace meda
