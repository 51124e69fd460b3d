// Device-side helpers shared by the gfx950 kernels of libtorq.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace torq {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(8 * sizeof(int)))) int i32x8;
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short i16x4;

// ---------------------------------------------------------------------------
// MXFP4 quantiser for one microscaling block (Section 4, Eq. 1; Algorithm 3,
// step 4).  The shared scale is the E8M0 byte with 2^(byte-127) =
// 2^(floor(log2 amax) - 2): for a normal fp32 amax that is the exponent field
// minus 2, clamped at 0 (amax is finite, so the field is at most 254).

__device__ __forceinline__ uint32_t e8m0_from_amax(float amax) {
  int field = (int)((__float_as_uint(amax) >> 23) & 0xFFu);
  int b = field - 2;
  return (uint32_t)(b < 0 ? 0 : b);
}

// 2^(byte-127) as an fp32 value; byte 0 is the subnormal 2^-127.
__device__ __forceinline__ float e8m0_to_f32(uint32_t byte) {
  return __uint_as_float(byte ? (byte << 23) : 0x00400000u);
}

// Eight consecutive elements of a block -> eight e2m1 nibbles in one dword,
// element 0 in the lowest nibble.  v_cvt_scalef32_pk_fp4_f32 divides its two
// inputs by `scale`, rounds to the nearest e2m1 value with ties to the even
// code, saturates at 6, keeps the sign bit, and writes one byte of the result.
__device__ __forceinline__ uint32_t pack8_e2m1(const float z[8], float scale) {
  uint32_t r = 0;
  r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, z[0], z[1], scale, 0);
  r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, z[2], z[3], scale, 1);
  r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, z[4], z[5], scale, 2);
  r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, z[6], z[7], scale, 3);
  return r;
}

__device__ __forceinline__ float amax8(const float z[8]) {
  float a = fmaxf(fmaxf(fabsf(z[0]), fabsf(z[1])), fabsf(z[2]));
  a = fmaxf(fmaxf(a, fabsf(z[3])), fabsf(z[4]));
  a = fmaxf(fmaxf(a, fabsf(z[5])), fabsf(z[6]));
  return fmaxf(a, fabsf(z[7]));
}

// ---------------------------------------------------------------------------
// The other 4-bit block formats of Section 6 ("Generalizability to Other Formats").  The paper names
// them without defining them; the readings are those of include/torq.h.

constexpr int FMT_NONE = -1, FMT_MXFP4 = 0, FMT_MXINT4 = 1, FMT_NVFP4 = 2;

// MXINT4: eight values -> eight two's-complement nibbles.  inv_scale = 2^(127 - byte) (the product is
// exact), round to nearest even, clamp to [-7, 7].
__device__ __forceinline__ float e8m0_inverse_f32(uint32_t byte) {   // byte <= 252 for finite input
  return __uint_as_float((254u - byte) << 23);
}
// Adding 1.5 * 2^23 rounds a small value to the nearest integer, ties to even, leaving it in two's
// complement in the low mantissa bits; the product with a power of two is exact, so one fused
// multiply-add rounds exactly what a multiply followed by that add would.  Clamping to [-7, 7] commutes
// with the rounding (the bounds are integers) and is done on the sum.
__device__ __forceinline__ uint32_t pack8_int4(const float z[8], float inv_scale) {
  uint32_t r = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float t = __builtin_amdgcn_fmed3f(__builtin_fmaf(z[i], inv_scale, 12582912.0f), 12582905.0f, 12582919.0f);
    r |= (__float_as_uint(t) & 15u) << (4 * i);
  }
  return r;
}

// OCP FP8 E4M3 (bias 7, largest value 448 = 0x7E, 0x7F is NaN) of t >= 0: round to nearest even
// on three mantissa bits, saturating.  Below 2^-6 the codes are the multiples of 2^-9.
__device__ __forceinline__ uint32_t e4m3_from_f32(float t) {
  if (t < 0.015625f) return (uint32_t)rintf(t * 512.0f);          // 0 .. 8; 8 is the first normal
  uint32_t u = __float_as_uint(t);
  u += 0x7FFFFu + ((u >> 20) & 1u);
  const uint32_t code = (u >> 20) - (120u << 3);
  return code < 0x7Eu ? code : 0x7Eu;
}
__device__ __forceinline__ float e4m3_to_f32(uint32_t code) {     // code <= 0x7E
  return (code >> 3) ? __uint_as_float(((code >> 3) + 120u) << 23 | (code & 7u) << 20)
                     : (float)code * 0.001953125f;
}
// NVFP4's block scale: the E4M3 code of amax / (6 * tensor scale), an IEEE division by definition.  As in
// pack8_nvfp4 below the division is carried out only where it can matter: the conversion is monotone, so
// where both ends of a bracket around the quotient convert to the same code the quotient does too.
__device__ __forceinline__ uint32_t nvfp4_scale_code(float amax, float six_gs) {
  if (six_gs >= 0x1p-100f && six_gs <= 0x1p100f) {
    const float t = amax * __builtin_amdgcn_rcpf(six_gs);
    const uint32_t lo = e4m3_from_f32(t * 0.99999904632568359375f), hi = e4m3_from_f32(t * 1.00000095367431640625f);
    if (lo == hi) return lo;
  }
  return e4m3_from_f32(__fdiv_rn(amax, six_gs));
}

// NVFP4: eight values of a block with effective scale S = e4m3 value * tensor scale.  IEEE
// division, then the e2m1 rounding of pack8_e2m1; a block whose scale rounded to zero keeps signs.
// The division is only carried out where it can matter.  With r = 1 / S to one ulp, a = z r is within
// 2^-22 (relative) of the IEEE quotient q, so a (1 - 2^-20) <= q <= a (1 + 2^-20) in magnitude; the e2m1
// rounding is monotone, so where both ends of that bracket round to the same code q does as well, and it
// is the code of a.  Otherwise (a quotient within 2^-20 of a rounding boundary, ties among them: a few
// values in a million) the lane divides.  S outside [2^-100, 2^100]: always divides.
__device__ __forceinline__ uint32_t pack8_nvfp4(const float z[8], float S) {
  float a[8];
  if (S >= 0x1p-100f && S <= 0x1p100f) {
    const float r = __builtin_amdgcn_rcpf(S);
    float lo[8], hi[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      a[i] = z[i] * r;
      lo[i] = a[i] * 0.99999904632568359375f;      // 1 - 2^-20
      hi[i] = a[i] * 1.00000095367431640625f;      // 1 + 2^-20
    }
    const uint32_t c = pack8_e2m1(a, 1.0f);
    if (pack8_e2m1(lo, 1.0f) == pack8_e2m1(hi, 1.0f)) return c;
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = (S > 0.0f) ? __fdiv_rn(z[i], S) : copysignf(0.0f, z[i]);
  return pack8_e2m1(a, 1.0f);
}

// bf16 <-> fp32 bit moves
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

}  // namespace torq
