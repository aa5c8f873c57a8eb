// paged_decode_attn kernels (gfx950): decode attention (Section 2) over the quantized paged
// cache (Section 7.2.2).  Two launches: a split kernel over (sequence, kv head, chunk) that
// streams K/V codes from HBM once, and a small log-sum-exp reduce over the chunks.
//
// Split kernel, per 64-lane wavefront and per 64-token group (four 16-token sub-blocks):
//   * K codes: lane (m = lane%16, c = lane/16) loads 16-byte pieces of token
//     (sub-block m/4, token 4u + m%4) for u = 0..3, channels [64j + 16c, +16).
//     That is directly the A operand (M = 16 tokens, K = 32 channels per instruction) of
//     v_mfma_f32_16x16x32_f16; q (f16, loaded once) is the B operand with the G*q_len query
//     rows that share the kv head as the N columns.  The accumulator then holds, in lane
//     (row n = lane%16, g = lane/16), the logits of the 16 tokens of sub-block g.
//   * V codes are stored channel-major, so lane (m, g) loads 16 bytes = 16 tokens of
//     sub-block g for channel 16t + m: the A operand (M = 16 channels, K = tokens) of the
//     P.V instruction, whose B operand is exactly the lane's own 16 probabilities.  No
//     shuffle, LDS transpose or re-layout sits between the two contractions.
//   * Codes become f16 exactly (int8: magic-number bytes; e4m3: exponent re-bias by shifting,
//     which leaves a factor 2^8 that is folded into the scale), the K scale multiplies the
//     logit after the contraction and the V scale is folded into the probability.
//   * Online softmax in base 2.  The running reference m is the maximum of
//     (logit + log2 V-scale), so the f16 probabilities p*sV stay in (0, 2^10] whatever the
//     magnitude of V; the plain softmax denominator is recovered as sum(P * 2^-lsv).
//   * The four wavefronts of a workgroup take the chunk's groups round-robin and merge their
//     (m, l, acc) through LDS; the workgroup writes one partial, or the final rows when the
//     sequence has a single chunk.
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

constexpr int kWaves = 4;
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
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x150 + I, 0xF, 0xF, false));
}

__device__ inline float xor16_max(float v) {
  v = fmaxf(v, __shfl_xor(v, 16, 64));
  return fmaxf(v, __shfl_xor(v, 32, 64));
}
__device__ inline float xor16_sum(float v) {
  v += __shfl_xor(v, 16, 64);
  return v + __shfl_xor(v, 32, 64);
}

// Four code bytes (one dword) -> four f16, in byte order.
template <int MODE>
__device__ inline void cvt4(uint32_t x, half2v& lo, half2v& hi) {
  if constexpr (MODE == KVQ_INT8_TOKEN_HEAD) {
    // byte b (two's complement) ^ 0x80 = b + 128 as unsigned; 0x6400 | u is the f16 1024 + u
    const uint32_t y = x ^ 0x80808080u;
    const uint32_t a = __builtin_amdgcn_perm(0x64646464u, y, 0x04010400u);
    const uint32_t b = __builtin_amdgcn_perm(0x64646464u, y, 0x04030402u);
    const half2v bias = {(_Float16)1152.0f, (_Float16)1152.0f};
    lo = __builtin_bit_cast(half2v, a) - bias;
    hi = __builtin_bit_cast(half2v, b) - bias;
  } else {
    // S.EEEE.MMM placed as S.0EEEE.MMM0000000: the f16 with value e4m3 * 2^-8 (subnormals too)
    const uint32_t a = __builtin_amdgcn_perm(0u, x, 0x010c000cu);  // (b1 << 24) | (b0 << 8)
    const uint32_t b = __builtin_amdgcn_perm(0u, x, 0x030c020cu);  // (b3 << 24) | (b2 << 8)
    const short2v one = {1, 1};
    const uint32_t sa = __builtin_bit_cast(uint32_t, __builtin_bit_cast(short2v, a) >> one);
    const uint32_t sb = __builtin_bit_cast(uint32_t, __builtin_bit_cast(short2v, b) >> one);
    lo = __builtin_bit_cast(half2v, sa & 0xBFFFBFFFu);
    hi = __builtin_bit_cast(half2v, sb & 0xBFFFBFFFu);
  }
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

template <int MODE, int D, int NT>
__global__ __launch_bounds__(kWaves * 64) void attn_split_kernel(const AttnArgs p) {
  constexpr int DT = D / 16;
  constexpr int KJ = D / 64;
  constexpr int KS = D / 32;  // MFMA steps over the channels
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m16 = lane & 15, g4 = lane >> 4;

  int id = blockIdx.x;
  const int c = id % p.num_chunks;
  id /= p.num_chunks;
  const int h = id % p.num_kv_heads;
  id /= p.num_kv_heads;
  const int rg = id % p.num_row_groups;
  const int b = id / p.num_row_groups;

  const int L = p.seq_lens[b];
  const int start = c * p.chunk_tokens;
  if (start >= L) return;
  const int end = min(start + p.chunk_tokens, L);
  const int ngroups = (end - start + 63) >> 6;
  const int last_sb = ((L - 1) >> 4) << 4;  // first position of the last 16-token sub-block
  const int bs = p.block_size, bs_shift = p.bs_shift, H = p.num_kv_heads;
  const int32_t* __restrict__ table = p.block_tables + (size_t)b * p.max_blocks_per_seq;
  const uint8_t* __restrict__ cache = p.cache;
  const float* __restrict__ scales = p.scales;
  const size_t tile_bytes = (size_t)bs * D;

  // ---- q: B operand of the QK^T instruction, and each row's causal length ----
  half8 qb[NT][KS];
  int nrow[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int r = (rg * NT + nt) * 16 + m16;
    const bool live = r < p.rows;
    const int j = live ? r / p.group : 0;
    const int gi = live ? r - j * p.group : 0;
    nrow[nt] = live ? L - p.q_len + j + 1 : L;
    const uint16_t* qrow =
        p.q + (((size_t)b * p.q_len + j) * p.num_q_heads + (size_t)h * p.group + gi) * D;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const int d0 = 64 * (s >> 1) + 16 * g4 + 8 * (s & 1);
      const uintx4 raw = *(const uintx4*)(qrow + d0);
      half8 x;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        x[2 * e] = (_Float16)__uint_as_float(raw[e] << 16);
        x[2 * e + 1] = (_Float16)__uint_as_float(raw[e] & 0xFFFF0000u);
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) qb[nt][s][e] = live ? x[e] : (_Float16)0.0f;
    }
  }

  // ---- running state ----
  floatx4 acc[NT][DT];
  float m_run[NT], l_run[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    m_run[nt] = -INFINITY;
    l_run[nt] = 0.0f;
#pragma unroll
    for (int t = 0; t < DT; ++t) acc[nt][t] = floatx4{0.f, 0.f, 0.f, 0.f};
  }

  // per-lane constants of the address arithmetic
  const int sbk = m16 >> 2;                                   // sub-block this lane reads K from
  const uint32_t block_stride = 2u * (uint32_t)H * (uint32_t)tile_bytes;  // bytes per cache block
  const uint32_t k_lane = (uint32_t)h * (uint32_t)tile_bytes + (uint32_t)(m16 & 3) * D + 16u * g4;
  const uint32_t v_lane = ((uint32_t)H + (uint32_t)h) * (uint32_t)tile_bytes + (uint32_t)m16 * bs;
  const uint32_t s_block_stride = (MODE == KVQ_INT8_TOKEN_HEAD) ? 2u * H * bs : 2u * H;
  const uint32_t s_lane = (MODE == KVQ_INT8_TOKEN_HEAD) ? (uint32_t)h * bs + m16 : (uint32_t)h;
  const uint32_t s_kv = (MODE == KVQ_INT8_TOKEN_HEAD) ? (uint32_t)H * bs : (uint32_t)H;

  // block-table entries of the sub-blocks this lane reads K and V from
  auto fetch_entries = [&](int gidx, int& blk_k, int& blk_v) {
    const int pos0 = start + (gidx << 6);
    blk_k = table[min(pos0 + 16 * sbk, last_sb) >> bs_shift];
    blk_v = table[min(pos0 + 16 * g4, last_sb) >> bs_shift];
  };

  // K codes and both scales of a group; also works out where the group's V codes are
  auto load_k = [&](uintx4 (&kt)[4][KJ], float& sk, float& sv, const uint8_t*& vbase, int gidx,
                    int blk_k, int blk_v) {
    const int pos0 = start + (gidx << 6);
    const uint32_t off_k = (uint32_t)(min(pos0 + 16 * sbk, last_sb) & (bs - 1));
    const uint32_t off_v = (uint32_t)(min(pos0 + 16 * g4, last_sb) & (bs - 1));
    const uint8_t* kbase = cache + (size_t)blk_k * block_stride + (off_k * D + k_lane);
    vbase = cache + (size_t)blk_v * block_stride + (v_lane + off_v);
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int j = 0; j < KJ; ++j) kt[u][j] = *(const uintx4*)(kbase + u * 4 * D + 64 * j);
    const float* sp = scales + (size_t)blk_v * s_block_stride +
                      (s_lane + (MODE == KVQ_INT8_TOKEN_HEAD ? off_v : 0u));
    sk = sp[0];
    sv = sp[s_kv];
  };
  auto load_v = [&](uintx4 (&vt)[DT], const uint8_t* vbase) {
#pragma unroll
    for (int tt = 0; tt < DT; ++tt) vt[tt] = *(const uintx4*)(vbase + (size_t)tt * 16 * bs);
  };

  // ---- S^T = K q^T ----
  auto qk = [&](const uintx4 (&kt)[4][KJ], floatx4 (&S)[NT][4]) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int u = 0; u < 4; ++u) S[nt][u] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int j = 0; j < KJ; ++j) {
        const uintx4 raw = kt[u][j];
        const half8 a0 = cvt8<MODE>(raw[0], raw[1]);
        const half8 a1 = cvt8<MODE>(raw[2], raw[3]);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          S[nt][u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, qb[nt][2 * j], S[nt][u], 0, 0, 0);
          S[nt][u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, qb[nt][2 * j + 1], S[nt][u], 0, 0, 0);
        }
      }
  };

  // ---- online softmax of a group: S (logits) -> pb (f16 probabilities x V scale) ----
  auto softmax = [&](floatx4 (&S)[NT][4], float sk, float sv, int gidx, half8 (&pb)[NT][2]) {
    const int pos0 = start + (gidx << 6);
    // a group is a "tail" if some row's causal length ends inside it
    const bool tail = pos0 + 64 > L - p.q_len + 1;
    // this lane's scales: logit factor, log2 of the V scale and its inverse
    const float fold = (MODE == KVQ_FP8E4M3_BLOCK_HEAD) ? 256.0f : 1.0f;  // 2^8 of the f16 trick
    float skp = sk * (p.scale_log2 * fold);
    float lsv = __builtin_amdgcn_logf(fmaxf(sv * fold, kMinVScale));
    float rsv = __builtin_amdgcn_exp2f(-lsv);
    if (MODE == KVQ_INT8_TOKEN_HEAD && tail && pos0 + 16 * g4 + m16 >= L) {
      skp = 0.0f;  // a slot that was never written: its scales are not data
      lsv = 0.0f;
      rsv = 0.0f;
    }
    // logits in base 2, shifted by log2 of the V scale; row maximum
    float mx[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) mx[nt] = -INFINITY;
    static_for<16>([&](auto I) {
      constexpr int tix = decltype(I)::value, u = tix >> 2, i = tix & 3;
      float ks, ls;
      if constexpr (MODE == KVQ_INT8_TOKEN_HEAD) {
        ks = row_bcast<tix>(skp);
        ls = row_bcast<tix>(lsv);
      } else {
        ks = skp;
        ls = lsv;
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        float ze = S[nt][u][i] * ks + ls;
        if (tail) ze = (pos0 + 16 * g4 + tix < nrow[nt]) ? ze : -INFINITY;
        S[nt][u][i] = ze;
        mx[nt] = fmaxf(mx[nt], ze);
      }
    });
    bool rescale = false;
    float alpha[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const float m_new = fmaxf(m_run[nt], xor16_max(mx[nt]));
      const float m_safe = (m_new == -INFINITY) ? 0.0f : m_new;
      alpha[nt] = __builtin_amdgcn_exp2f(m_run[nt] - m_safe);
      rescale |= (alpha[nt] != 1.0f);
      m_run[nt] = m_new;
      const float msub = m_safe - kPOffset;
      float lsum = 0.0f;
      static_for<16>([&](auto I) {
        constexpr int tix = decltype(I)::value, u = tix >> 2, i = tix & 3;
        const float pr = __builtin_amdgcn_exp2f(S[nt][u][i] - msub);
        float rs;
        if constexpr (MODE == KVQ_INT8_TOKEN_HEAD) rs = row_bcast<tix>(rsv);
        else rs = rsv;
        lsum += pr * rs;
        pb[nt][tix >> 3][tix & 7] = (_Float16)pr;
      });
      l_run[nt] = l_run[nt] * alpha[nt] + lsum;
    }
    if (__any(rescale)) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int tt = 0; tt < DT; ++tt) acc[nt][tt] *= alpha[nt];
    }
  };

  // ---- acc^T += V^T P^T ----
  auto pv = [&](const uintx4 (&vt)[DT], const half8 (&pb)[NT][2]) {
#pragma unroll
    for (int tt = 0; tt < DT; ++tt) {
      const uintx4 raw = vt[tt];
      const half8 a0 = cvt8<MODE>(raw[0], raw[1]);
      const half8 a1 = cvt8<MODE>(raw[2], raw[3]);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        acc[nt][tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, pb[nt][0], acc[nt][tt], 0, 0, 0);
        acc[nt][tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, pb[nt][1], acc[nt][tt], 0, 0, 0);
      }
    }
  };

  // ---- main loop: this wave takes groups wave, wave + 4, ...  K and V each live in one
  // register buffer: the next group's K codes are requested as soon as QK^T has consumed the
  // current ones, the next V codes as soon as P.V has, so loads stay in flight behind the
  // arithmetic; block-table entries are fetched one group further ahead ----
  if (wave < ngroups) {
    uintx4 kt[4][KJ], vt[DT];
    float sk, sv;
    const uint8_t* vbase;
    int blk_k, blk_v;
    int g = wave;
    // The table entries of a group are requested one group ahead and always before the
    // loads that follow them in program order (here: both requests first, then the codes), so
    // that waiting for an entry never waits for code loads issued behind it.
    {
      int bk0, bv0;
      fetch_entries(g, bk0, bv0);
      fetch_entries(min(g + kWaves, ngroups - 1), blk_k, blk_v);
      __builtin_amdgcn_sched_barrier(0);
      load_k(kt, sk, sv, vbase, g, bk0, bv0);
      load_v(vt, vbase);
    }
    floatx4 S[NT][4];
    half8 pb[NT][2];
    for (; g + kWaves < ngroups; g += kWaves) {  // steady state: a next group exists
      const int gn = g + kWaves;
      qk(kt, S);
      const float sk_cur = sk, sv_cur = sv;
      load_k(kt, sk, sv, vbase, gn, blk_k, blk_v);
      fetch_entries(min(gn + kWaves, ngroups - 1), blk_k, blk_v);
      softmax(S, sk_cur, sv_cur, g, pb);
      pv(vt, pb);
      load_v(vt, vbase);
    }
    qk(kt, S);  // the wave's last group: nothing left to request
    softmax(S, sk, sv, g, pb);
    pv(vt, pb);
  }

  // ---- merge the four waves through LDS ----
  constexpr int RS = D + 4;  // padded row stride (floats)
  __shared__ float sm_m[kWaves][NT * 16];
  __shared__ float sm_l[kWaves][NT * 16];
  __shared__ float sm_acc[kWaves - 1][NT * 16][RS];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    l_run[nt] = xor16_sum(l_run[nt]);
    if (g4 == 0) {
      sm_m[wave][nt * 16 + m16] = m_run[nt];
      sm_l[wave][nt * 16 + m16] = l_run[nt];
    }
  }
  __syncthreads();
  float m_all[NT], l_all[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    float mm = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) mm = fmaxf(mm, sm_m[w][nt * 16 + m16]);
    const float mm_safe = (mm == -INFINITY) ? 0.0f : mm;
    float ll = 0.0f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w)
      ll += sm_l[w][nt * 16 + m16] * __builtin_amdgcn_exp2f(sm_m[w][nt * 16 + m16] - mm_safe);
    const float f = __builtin_amdgcn_exp2f(m_run[nt] - mm_safe);
    m_all[nt] = mm;
    l_all[nt] = ll;
#pragma unroll
    for (int tt = 0; tt < DT; ++tt) acc[nt][tt] *= f;
    if (wave > 0) {
#pragma unroll
      for (int tt = 0; tt < DT; ++tt)
        *(floatx4*)&sm_acc[wave - 1][nt * 16 + m16][16 * tt + 4 * g4] = acc[nt][tt];
    }
  }
  __syncthreads();
  if (wave != 0) return;

  const int chunks_of_seq = (L + p.chunk_tokens - 1) / p.chunk_tokens;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int r = (rg * NT + nt) * 16 + m16;
#pragma unroll
    for (int tt = 0; tt < DT; ++tt)
#pragma unroll
      for (int w = 0; w < kWaves - 1; ++w)
        acc[nt][tt] += *(const floatx4*)&sm_acc[w][nt * 16 + m16][16 * tt + 4 * g4];
    if (r >= p.rows) continue;
    if (chunks_of_seq == 1) {
      const int j = r / p.group, gi = r - j * p.group;
      float* orow =
          p.out + (((size_t)b * p.q_len + j) * p.num_q_heads + (size_t)h * p.group + gi) * D;
      const float inv = 1.0f / l_all[nt];
#pragma unroll
      for (int tt = 0; tt < DT; ++tt) *(floatx4*)(orow + 16 * tt + 4 * g4) = acc[nt][tt] * inv;
    } else {
      const size_t item = (((size_t)b * H + h) * p.num_chunks + c) * p.rows + r;
      float* arow = p.ws_acc + item * D;
#pragma unroll
      for (int tt = 0; tt < DT; ++tt) *(floatx4*)(arow + 16 * tt + 4 * g4) = acc[nt][tt];
      if (g4 == 0) {
        p.ws_ml[item * 2] = m_all[nt];
        p.ws_ml[item * 2 + 1] = l_all[nt];
      }
    }
  }
}

// ---- log-sum-exp merge of the chunk partials: one workgroup per (sequence, query token,
// query head), one thread per channel ----
template <int D>
__global__ __launch_bounds__(D) void attn_reduce_kernel(const AttnArgs p) {
  int id = blockIdx.x;
  const int hq = id % p.num_q_heads;
  id /= p.num_q_heads;
  const int j = id % p.q_len;
  const int b = id / p.q_len;
  const int L = p.seq_lens[b];
  const int nc = (L + p.chunk_tokens - 1) / p.chunk_tokens;
  if (nc <= 1) return;  // the split kernel already wrote the final rows
  const int h = hq / p.group;
  const int r = j * p.group + (hq - h * p.group);
  const int d = threadIdx.x;
  const size_t item0 = (((size_t)b * p.num_kv_heads + h) * p.num_chunks) * p.rows + r;
  float M = -INFINITY;
  for (int c = 0; c < nc; ++c) M = fmaxf(M, p.ws_ml[(item0 + (size_t)c * p.rows) * 2]);
  float num = 0.0f, den = 0.0f;
  for (int c = 0; c < nc; ++c) {
    const size_t item = item0 + (size_t)c * p.rows;
    const float w = __builtin_amdgcn_exp2f(p.ws_ml[item * 2] - M);
    num += w * p.ws_acc[item * D + d];
    den += w * p.ws_ml[item * 2 + 1];
  }
  p.out[(((size_t)b * p.q_len + j) * p.num_q_heads + hq) * D + d] = num / den;
}

// measurement hook: events recorded around the split kernel (see kvq_profile_split_events)
hipEvent_t g_ev_before = nullptr, g_ev_after = nullptr;

template <int MODE, int D>
hipError_t launch_split(const AttnArgs& a, unsigned grid, hipStream_t stream) {
  if (g_ev_before) (void)hipEventRecord(g_ev_before, stream);
  if (a.row_tiles == 1)
    hipLaunchKernelGGL((attn_split_kernel<MODE, D, 1>), dim3(grid), dim3(kWaves * 64), 0, stream, a);
  else
    hipLaunchKernelGGL((attn_split_kernel<MODE, D, 2>), dim3(grid), dim3(kWaves * 64), 0, stream, a);
  const hipError_t e = hipGetLastError();
  if (g_ev_after) (void)hipEventRecord(g_ev_after, stream);
  return e;
}

}  // namespace

void set_profile_events(hipEvent_t before, hipEvent_t after) {
  g_ev_before = before;
  g_ev_after = after;
}

hipError_t launch_attn(const AttnArgs& a, hipStream_t stream) {
  const unsigned grid =
      (unsigned)((size_t)a.batch * a.num_row_groups * a.num_kv_heads * a.num_chunks);
  hipError_t e;
  if (a.mode == KVQ_INT8_TOKEN_HEAD)
    e = a.head_dim == 128 ? launch_split<KVQ_INT8_TOKEN_HEAD, 128>(a, grid, stream)
                          : launch_split<KVQ_INT8_TOKEN_HEAD, 64>(a, grid, stream);
  else
    e = a.head_dim == 128 ? launch_split<KVQ_FP8E4M3_BLOCK_HEAD, 128>(a, grid, stream)
                          : launch_split<KVQ_FP8E4M3_BLOCK_HEAD, 64>(a, grid, stream);
  if (e != hipSuccess) return e;
  if (a.num_chunks > 1) {
    const unsigned rgrid = (unsigned)((size_t)a.batch * a.q_len * a.num_q_heads);
    if (a.head_dim == 128)
      hipLaunchKernelGGL((attn_reduce_kernel<128>), dim3(rgrid), dim3(128), 0, stream, a);
    else
      hipLaunchKernelGGL((attn_reduce_kernel<64>), dim3(rgrid), dim3(64), 0, stream, a);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace kvq
