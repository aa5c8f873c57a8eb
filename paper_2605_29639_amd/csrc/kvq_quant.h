// Rounding of the int8 per-(token, head) format (Section 7.2.2), shared by the write kernels.
// Every path through these functions yields the nearest integer (ties to even) of the exact
// quotient x / s.
#pragma once
#include "kvq_internal.h"

namespace kvq {

__device__ inline float bf16_bits_to_float(uint32_t bits16) {
  return __uint_as_float(bits16 << 16);
}

// The scale of a row whose largest |x| has the bf16 bit pattern amax_bits: absmax / 127 rounded
// once to fp32 (a correctly rounded fp32 division equals the fp64 quotient rounded once for
// every bf16 absmax).
__device__ inline float int8_scale(uint32_t amax_bits) {
  return amax_bits == 0 ? 0.0f : __fdiv_rn(bf16_bits_to_float(amax_bits), 127.0f);
}

// fp64 quotient: either exactly a tie or at least 2^-25 away from one for a bf16 x and an fp32
// s, so rounding it equals rounding the exact quotient.
__device__ inline uint8_t int8_code(float x, float s) {
  double r = rint((double)x / (double)s);  // v_rndne_f64: ties to even
  r = r > 127.0 ? 127.0 : r;
  r = r < -127.0 ? -127.0 : r;
  return (uint8_t)(int8_t)(int)r;
}

// The same code as a float, through fp32 where that is safe: x * rcp(s) is within 2.3e-5 of the
// exact quotient (|quotient| <= 127, rcp within one ulp, one rounding for the product), so
// unless it lies within 4e-5 of a half-integer its nearest integer is the exact quotient's;
// the rare elements that do are decided in fp64.  `inv` = rcp(s) and `fast` = (s > 1e-30f, the
// reciprocal of a denormal is not usable) are the caller's, computed once per row.
__device__ inline float int8_code_f32(float x, float s, float inv, bool fast) {
  const float q = x * inv;
  float r = __builtin_rintf(q);
  if (__builtin_expect(!fast || fabsf(q - r) > 0.5f - 4e-5f, 0))
    r = (s == 0.0f) ? 0.0f : (float)(int8_t)int8_code(x, s);
  return r;
}

// Maximum over the CL (4, 8 or 16) adjacent lanes that share a row of 16.
template <int CL>
__device__ inline uint32_t row_max_u32(uint32_t v) {
  auto mx = [](uint32_t a, uint32_t b) { return a > b ? a : b; };
  v = mx(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
  v = mx(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
  if constexpr (CL >= 8)
    v = mx(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, false));  // row_half_mirror
  if constexpr (CL == 16)
    v = mx(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, false));  // row_mirror
  return v;
}

}  // namespace kvq
