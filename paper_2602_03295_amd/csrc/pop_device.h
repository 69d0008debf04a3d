// Small device-side helpers shared by the gfx950 kernels (bf16 packing, wave reductions).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pop {

constexpr int kWave = 64;  // CDNA wavefront width

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4_t;

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __builtin_bit_cast(float, (uint32_t)b << 16);
}
// round-to-nearest-even
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f));
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}
// fp16 (round-to-nearest-even, saturating instead of overflowing to infinity)
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8_t;
__device__ __forceinline__ uint16_t f32_to_f16_sat(float f) {
  const float c = fminf(fmaxf(f, -65504.f), 65504.f);
  return __builtin_bit_cast(uint16_t, static_cast<_Float16>(c));
}
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
  return (uint32_t)f32_to_f16_sat(lo) | ((uint32_t)f32_to_f16_sat(hi) << 16);
}
__device__ __forceinline__ float f16lo(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffff)); }
__device__ __forceinline__ float f16hi(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16)); }
__device__ __forceinline__ float bf16lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

// 8-bit floating point with 4 exponent bits (bias 7), 3 mantissa bits, no infinities ("e4m3", largest finite value
// 448, code 0x7f / 0xff = NaN), in software so that the rounding is the one written here whatever the hardware's
// conversion instructions implement: nearest value, ties to the even mantissa, magnitudes beyond 448 clamp to 448
// (a NaN input gives the NaN code).
__device__ __forceinline__ uint32_t e4m3_encode(float x) {
  const uint32_t bits = __builtin_bit_cast(uint32_t, x);
  const uint32_t sign = (bits >> 24) & 0x80u;
  float a = __builtin_fabsf(x);
  if (!(a == a)) return sign | 0x7fu;
  a = fminf(a, 448.f);
  uint32_t code;
  if (a < 0.015625f) {                       // below the smallest normal value 2^-6: steps of 2^-9
    code = (uint32_t)__builtin_rintf(a * 512.f);          // 0 .. 8 (8 is the code of 2^-6 itself)
  } else {
    uint32_t u = __builtin_bit_cast(uint32_t, a);
    u += 0x7ffffu + ((u >> 20) & 1u);        // round to nearest even at bit 20 (3 mantissa bits kept)
    code = ((u >> 20) & 0x7ffu) - ((127u - 7u) << 3);     // exponent re-biased from 127 to 7, mantissa below it
  }
  return sign | code;
}
__device__ __forceinline__ float e4m3_decode(uint32_t c) {
  const uint32_t mag = c & 0x7fu;
  // normal: exponent field e = mag >> 3 (>= 1), value (1 + m / 8) 2^(e - 7); subnormal: m 2^-9
  const float normal = __builtin_bit_cast(float, (mag << 20) + ((127u - 7u) << 23));
  const float sub = (float)mag * 0.001953125f;
  const float v = mag < 8u ? sub : normal;
  return (c & 0x80u) ? -v : v;
}
// Four codes of one 32-bit word -> four floats with the hardware's conversion (v_cvt_pk_f32_fp8; gfx950 reads the
// codes as this same format).  Decoding is exact, so there is no rounding to choose: checked on the device against
// e4m3_decode for all 254 codes that are numbers; the two NaN codes give NaN here (e4m3_decode returns 480 for them;
// they are never stored from a number).  A quarter of the instructions of the software form, which is what the
// decode attention over an 8-bit cache spends its time on.
__device__ __forceinline__ void e4m3_decode4_hw(uint32_t w, float* f) {
  typedef float f2_t __attribute__((ext_vector_type(2)));
  const f2_t lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false), hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
  f[0] = lo.x; f[1] = lo.y; f[2] = hi.x; f[3] = hi.y;
}
// Four values -> four codes in one 32-bit word (element 0 in the low byte).
__device__ __forceinline__ uint32_t e4m3_pack4(float a, float b, float c, float d) {
  return e4m3_encode(a) | (e4m3_encode(b) << 8) | (e4m3_encode(c) << 16) | (e4m3_encode(d) << 24);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Data-parallel-primitive moves inside a row of 16 lanes: no trip through LDS, unlike __shfl_xor.
// CTRL: 0xB1 = quad_perm [1,0,3,2], 0x4E = quad_perm [2,3,0,1], 0x141 = row_half_mirror (lane i <-> 7 - i of
// each 8), 0x140 = row_mirror (lane i <-> 15 - i of each 16).
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
// Sum / maximum over each aligned group of N consecutive lanes (N = 2, 4, 8, 16); every lane of the group
// receives the same bits.
template <int N>
__device__ __forceinline__ float group_sum(float v) {
  static_assert(N == 2 || N == 4 || N == 8 || N == 16, "group inside a row of 16 lanes");
  v += dpp_f32<0xB1>(v);
  if (N >= 4) v += dpp_f32<0x4E>(v);
  if (N >= 8) v += dpp_f32<0x141>(v);
  if (N >= 16) v += dpp_f32<0x140>(v);
  return v;
}
template <int N>
__device__ __forceinline__ float group_max(float v) {
  static_assert(N == 2 || N == 4 || N == 8 || N == 16, "group inside a row of 16 lanes");
  v = fmaxf(v, dpp_f32<0xB1>(v));
  if (N >= 4) v = fmaxf(v, dpp_f32<0x4E>(v));
  if (N >= 8) v = fmaxf(v, dpp_f32<0x141>(v));
  if (N >= 16) v = fmaxf(v, dpp_f32<0x140>(v));
  return v;
}
// Whole-wave forms: the four steps inside the rows as above, the two across rows through __shfl_xor.
__device__ __forceinline__ float wave_sum_rows(float v) {
  v = group_sum<16>(v);
  v += __shfl_xor(v, 16, 64);
  return v + __shfl_xor(v, 32, 64);
}
__device__ __forceinline__ float wave_max_rows(float v) {
  v = group_max<16>(v);
  v = fmaxf(v, __shfl_xor(v, 16, 64));
  return fmaxf(v, __shfl_xor(v, 32, 64));
}

}  // namespace pop
