// Device-side helpers shared by the gfx950 kernels: bf16 packing, exact RoPE phase,
// sin/cos on a reduced argument.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ba_internal.h"

namespace ba {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// two floats -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2_t f = {lo, hi};
  bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
  return __builtin_bit_cast(uint32_t, b);
}

__device__ __forceinline__ uint32_t fast_div(uint32_t n, const FastDiv &f) {
  const uint32_t t = __umulhi(n, f.mul);
  return (t + ((n - t) >> f.sh1)) >> f.sh2;
}

// two floats -> packed fp16 pair, round to nearest even; and back
__device__ __forceinline__ uint32_t pack_f16(float lo, float hi) {
  typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
  f32x2_t f = {lo, hi};
  f16x2_t h = __builtin_convertvector(f, f16x2_t);
  return __builtin_bit_cast(uint32_t, h);
}
__device__ __forceinline__ float f16_lo(uint32_t w) {
  typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
  return (float)__builtin_bit_cast(f16x2_t, w)[0];
}
__device__ __forceinline__ float f16_hi(uint32_t w) {
  typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
  return (float)__builtin_bit_cast(f16x2_t, w)[1];
}

// cos and sin of the angle whose fraction of a full turn is phase / 2^64.
// The quarter turn nearest to the phase is split off exactly in integer arithmetic;
// the remainder y, |y| <= pi/4, goes through Taylor polynomials whose truncation
// error is below 2e-9, so the result is accurate to about one fp32 ulp of 1.
__device__ __forceinline__ void sincos_phase(uint64_t phase, float &c, float &s) {
  uint32_t hi = (uint32_t)(phase >> 32);
  uint32_t quad = (hi + 0x20000000u) >> 30;     // nearest quarter turn, 0..3 (4 wraps to 0)
  int32_t rem = (int32_t)(hi - (quad << 30));   // signed remainder, Q0.32 turns
  float y = (float)rem * 1.4629180792671596e-9f;  // 2*pi / 2^32
  float y2 = y * y;
  float sp = -1.0f / 5040.0f + y2 * (1.0f / 362880.0f);
  sp = 1.0f / 120.0f + y2 * sp;
  sp = -1.0f / 6.0f + y2 * sp;
  float sy = y + y * y2 * sp;
  float cp = 1.0f / 40320.0f + y2 * (-1.0f / 3628800.0f);
  cp = -1.0f / 720.0f + y2 * cp;
  cp = 1.0f / 24.0f + y2 * cp;
  cp = -0.5f + y2 * cp;
  float cy = 1.0f + y2 * cp;
  quad &= 3u;
  float c0 = (quad & 1u) ? sy : cy;
  float s0 = (quad & 1u) ? cy : sy;
  c = (quad == 1u || quad == 2u) ? -c0 : c0;
  s = (quad >= 2u) ? -s0 : s0;
}

// phase of position * theta_j; position may be negative (two's complement wraps).
__device__ __forceinline__ uint64_t rope_phase(int32_t position, uint64_t turns) {
  return (uint64_t)(int64_t)position * turns;
}

}  // namespace ba
