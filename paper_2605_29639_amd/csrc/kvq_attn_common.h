// Device helpers shared by the attention kernels (kvq_attn.hip, kvq_prefill.hip): vector
// types, stored codes -> f16, the cross-lane pieces of the softmax.
#pragma once

#include <utility>

#include "kvq_internal.h"

namespace kvq {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef short short2v __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr float kPOffset = 10.0f;   // probabilities are scaled by 2^10 (cancels in acc / l)
constexpr float kMinVScale = 7.888609052210118e-31f;  // 2^-100

template <class F, int... Is>
__device__ inline void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
  (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ inline void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// value of lane I of the caller's 16-lane row
template <int I>
__device__ inline float row_bcast(float x) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x150 + I, 0xF, 0xF, true));
}

__device__ inline float xor16_max(float v) {
  v = fmaxf(v, __shfl_xor(v, 16, 64));
  return fmaxf(v, __shfl_xor(v, 32, 64));
}
__device__ inline float xor16_sum(float v) {
  v += __shfl_xor(v, 16, 64);
  return v + __shfl_xor(v, 32, 64);
}

// Four stored code bytes (one dword) -> four f16, in byte order.
template <int MODE>
__device__ inline void cvt4(uint32_t x, half2v& lo, half2v& hi) {
  if constexpr (MODE == KVQ_INT8_TOKEN_HEAD) {
    // stored byte u = code + 128; 0x6400 | u is the f16 1024 + u, so subtracting 1152 gives code
    const uint32_t a = __builtin_amdgcn_perm(0x64646464u, x, 0x04010400u);
    const uint32_t b = __builtin_amdgcn_perm(0x64646464u, x, 0x04030402u);
    const half2v bias = {(_Float16)1152.0f, (_Float16)1152.0f};
    lo = __builtin_bit_cast(half2v, a) - bias;
    hi = __builtin_bit_cast(half2v, b) - bias;
  } else {
    // gfx950's packed e4m3 -> f16 conversion (exact); NaN codes must not reach it as V data
    lo = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(x, 1.0f, false);
    hi = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(x, 1.0f, true);
  }
}

// Eight stored int4 nibbles (code + 8) of one word -> eight f16 codes; element 2i comes from
// nibble i, element 2i + 1 from nibble i + 4.  An AND-OR drops two nibbles, 16 bits apart,
// into the mantissas of a pair of f16 1024.0: nibbles at bits 0-3 give 1024 + n, nibbles at
// bits 4-7 give 1024 + 16 n; one packed add or fused multiply-add turns either into n - 8.
__device__ inline half8 cvt_int4(uint32_t x) {
  const half2v k1032 = {(_Float16)1032.0f, (_Float16)1032.0f};
  const half2v k16th = {(_Float16)0.0625f, (_Float16)0.0625f};
  const half2v k72 = {(_Float16)72.0f, (_Float16)72.0f};
  const uint32_t y = x >> 8;
  const half2v a = __builtin_bit_cast(half2v, (x & 0x000F000Fu) | 0x64006400u) - k1032;
  const half2v b = __builtin_bit_cast(half2v, (x & 0x00F000F0u) | 0x64006400u) * k16th - k72;
  const half2v c = __builtin_bit_cast(half2v, (y & 0x000F000Fu) | 0x64006400u) - k1032;
  const half2v d = __builtin_bit_cast(half2v, (y & 0x00F000F0u) | 0x64006400u) * k16th - k72;
  half8 r;
  r[0] = a[0]; r[1] = a[1]; r[2] = b[0]; r[3] = b[1];
  r[4] = c[0]; r[5] = c[1]; r[6] = d[0]; r[7] = d[1];
  return r;
}

template <int MODE>
__device__ inline half8 cvt8(uint32_t x0, uint32_t x1) {
  half2v a, b, c, d;
  cvt4<MODE>(x0, a, b);
  cvt4<MODE>(x1, c, d);
  half8 r;
  r[0] = a[0]; r[1] = a[1]; r[2] = b[0]; r[3] = b[1];
  r[4] = c[0]; r[5] = c[1]; r[6] = d[0]; r[7] = d[1];
  return r;
}

// Online softmax of one 64-token group for NT tiles of 16 query rows, shared by the streaming
// and the many-row kernels.  In: S, the raw contractions K.q in the accumulator layout (lane
// (row n, sub-block g) holds the 16 tokens of sub-block g); this lane's token's scales as
// skp = K scale * softmax scale * log2(e), lsv = log2(V scale), rsv = 1 / V scale (per token for
// the token-scaled formats, the same in every lane otherwise); pos_lane = position of the
// lane's first token; nrow = causal length of the lane's row per tile.  Out: pb, the
// probabilities times the V scale as the B operand of P.V (f16 scaled by 2^10, or two bf16
// terms for an unquantized cache) (for the group-scaled int4 format S is left holding those
// probabilities in fp32 instead); the running maximum m_run (of logit + lsv, base 2) and sum
// l_run are updated and acc is rescaled when a maximum moved.
// TAIL: some row's causal length ends inside the group, so positions are masked.
// The arithmetic on broadcast operands is kept as separate multiply / add so that the row
// broadcast rides on the instruction itself (v_mul_f32_dpp, v_add_f32_dpp) instead of costing
// moves.
template <int MODE, int NT, int DT, bool TAIL, class Operand, int NP>
__device__ inline void online_softmax(floatx4 (&S)[NT][4], float skp, float lsv, float rsv,
                                      int pos_lane, const int (&nrow)[NT], float (&m_run)[NT],
                                      float (&l_run)[NT], floatx4 (&acc)[NT][DT],
                                      Operand (&pb)[NT][NP]) {
#pragma clang fp contract(off)
  constexpr bool PLAIN = MODE == KVQ_BF16_PLAIN;
  constexpr bool FP8 = MODE == KVQ_FP8E4M3_BLOCK_HEAD || MODE == KVQ_FP8E4M3_TENSOR;
  constexpr bool TOKEN_SCALE = MODE == KVQ_INT8_TOKEN_HEAD || MODE == KVQ_INT4_TOKEN_HEAD ||
                               MODE == KVQ_INT4_GROUP32;
  // logits in base 2, shifted by log2 of the V scale; row maximum
  float mx[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) mx[nt] = -INFINITY;
  static_for<16>([&](auto I) {
    constexpr int tix = decltype(I)::value, u = tix >> 2, i = tix & 3;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      float ze;
      if constexpr (TOKEN_SCALE) {
        ze = S[nt][u][i] * row_bcast<tix>(skp);
        ze = ze + row_bcast<tix>(lsv);
      } else if constexpr (PLAIN) {
        ze = S[nt][u][i] * skp;
      } else {
        ze = __builtin_fmaf(S[nt][u][i], skp, lsv);
      }
      if constexpr (TAIL) ze = (pos_lane + tix < nrow[nt]) ? ze : -INFINITY;
      S[nt][u][i] = ze;
      mx[nt] = fmaxf(mx[nt], ze);
    }
  });
  float alpha[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const float m_new = fmaxf(m_run[nt], xor16_max(mx[nt]));
    const float m_safe = (m_new == -INFINITY) ? 0.0f : m_new;
    alpha[nt] = __builtin_amdgcn_exp2f(m_run[nt] - m_safe);
    m_run[nt] = m_new;
    const float msub = m_safe - kPOffset;
    float lsum = 0.0f;
    [[maybe_unused]] uint32_t hi_bits[16], lo_bits[16];
    static_for<16>([&](auto I) {
      constexpr int tix = decltype(I)::value, u = tix >> 2, i = tix & 3;
      const float pr = __builtin_amdgcn_exp2f(S[nt][u][i] - msub);
      if constexpr (MODE == KVQ_INT4_GROUP32) S[nt][u][i] = pr;  // its caller scales them once more
      if constexpr (TOKEN_SCALE) {
        lsum = __builtin_fmaf(pr, row_bcast<tix>(rsv), lsum);  // one v_fmac_f32_dpp
      } else {
        lsum = lsum + pr;
      }
      if constexpr (PLAIN) {
        // bf16 keeps 8 bits of a probability: it goes in as two terms, the value cut to
        // bf16 and the (exactly representable) rest cut to bf16, 16 bits in all
        hi_bits[tix] = __float_as_uint(pr) & 0xFFFF0000u;
        lo_bits[tix] = __float_as_uint(pr - __uint_as_float(hi_bits[tix]));
      } else {
        pb[nt][tix >> 3][tix & 7] = (_Float16)pr;
      }
    });
    if constexpr (PLAIN) {
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        uintx4 ph, pl;
#pragma unroll
        for (int e = 0; e < 4; ++e) {  // the upper halves of two tokens' words, packed
          ph[e] = __builtin_amdgcn_perm(hi_bits[8 * hf + 2 * e + 1], hi_bits[8 * hf + 2 * e], 0x07060302u);
          pl[e] = __builtin_amdgcn_perm(lo_bits[8 * hf + 2 * e + 1], lo_bits[8 * hf + 2 * e], 0x07060302u);
        }
        pb[nt][hf] = __builtin_bit_cast(bf16x8, ph);
        pb[nt][2 + hf] = __builtin_bit_cast(bf16x8, pl);
      }
    }
    if constexpr (FP8) lsum = lsum * rsv;  // one scale per lane
    l_run[nt] = l_run[nt] * alpha[nt] + lsum;
  }
  // (per 16-row tile: a tile none of whose rows' maxima moved keeps its accumulators as they are)
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    if (__any(alpha[nt] != 1.0f)) {
#pragma unroll
      for (int tt = 0; tt < DT; ++tt) acc[nt][tt] *= alpha[nt];
    }
  }
}

}  // namespace
}  // namespace kvq
