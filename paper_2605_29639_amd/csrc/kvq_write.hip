// kv_quant_write kernels (gfx950): bf16 K/V rows -> int8, int4 or fp8-e4m3 codes + fp32 scales
// in the paged cache (Section 7.2.2, on-the-fly quantization with dynamic scaling), or the
// rows themselves for an unquantized cache.
//
// One 64-lane wavefront owns one unit of work, so every output byte and every scale has
// exactly one writer and no atomics are needed:
//   int8 / int4 per (token, head): unit = (run, kv head, K|V), a run being consecutive tokens
//                           of the call with consecutive slots inside one 16-token sub-block;
//   fp8 per (block, head):  unit = (run, kv head, K|V), a run being the consecutive tokens
//                           of the call that fall into one cache block;
//   fp8 under static scales, bf16 rows: as int8 without the scale.
// Each format has a general routine (any run) and one for whole 16-token sub-blocks, which
// calls carrying a prompt take (16-byte loads, fp32 rounding with an fp64 decision near ties).
// The decisions that fix an integer (the rounding of x/scale) are taken in fp64: for a bf16
// x and an fp32 scale the fp64 quotient is either exactly a rounding tie or at least 2^-25
// (relative 2^-29 for the fp8 midpoints) away from one, so rounding it equals rounding the
// exact quotient.  The scale itself is the fp64 quotient absmax/qmax rounded once to fp32.
#include "kvq_quant.h"

namespace kvq {
namespace {

constexpr int kWaves = 4;  // wavefronts per workgroup
constexpr int kBulkTokens = 1024;  // calls with at least this many tokens take the prefill kernels

__device__ inline uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) {
    uint32_t o = (uint32_t)__shfl_xor((int)v, s, 64);
    v = v > o ? v : o;
  }
  return v;
}

// Nearest E4M3 (finite-only) code of the real y: ties to even, saturating at 448.
__device__ inline uint8_t fp8_code(double y) {
  const uint64_t bits = (uint64_t)__double_as_longlong(y);
  const uint32_t sign = (uint32_t)(bits >> 63) << 7;
  const double a = fabs(y);
  if (a >= 448.0) return (uint8_t)(sign | 0x7E);
  int e = (int)((bits >> 52) & 0x7FF) - 1023;  // floor(log2 a) for normal a
  e = e < -6 ? -6 : e;                         // below 2^-6 the spacing stays 2^-9
  const int r = (int)rint(ldexp(a, 3 - e));    // a / 2^(e-3), exact scaling; r in [0, 16]
  return (uint8_t)(sign | (uint32_t)(((e + 7) << 3) + r - 8));
}

__device__ inline double fp8_value(uint32_t c) {
  const int e = (c >> 3) & 15, m = c & 7;
  const double mag = e == 0 ? ldexp((double)m, -9) : ldexp((double)(8 + m), e - 10);
  return (c & 0x80) ? -mag : mag;
}

// A lane owns E = D/64 adjacent channels.  K bytes of a token for those channels are adjacent
// in the quad order (one 1- or 2-byte store).  V bytes of consecutive tokens for one channel
// are adjacent in the sub-block order, so a run of tokens is gathered per channel into one
// 16-byte row image and stored once: a whole sub-block as one 16-byte store per channel,
// a shorter run byte by byte (other slots of the row keep their contents).
struct RowImage {
  unsigned long long lo = 0, hi = 0;  // bytes 0..7 and 8..15 of a 16-token V row
  __device__ void put(int pos, uint8_t b) {
    if (pos < 8) lo |= (unsigned long long)b << (8 * pos);
    else hi |= (unsigned long long)b << (8 * (pos - 8));
  }
  __device__ uint8_t get(int pos) const {
    return (uint8_t)(pos < 8 ? lo >> (8 * pos) : hi >> (8 * (pos - 8)));
  }
};

// store bytes [first, first + n) of a 16-token V row
__device__ inline void store_v_row(uint8_t* row, const RowImage& img, int first, int n) {
  if (n == 16) {
    *(uint4*)row = make_uint4((uint32_t)img.lo, (uint32_t)(img.lo >> 32), (uint32_t)img.hi,
                              (uint32_t)(img.hi >> 32));
  } else {
    for (int j = first; j < first + n; ++j) row[j] = img.get(j);
  }
}

template <int E>
__device__ inline void store_k(uint8_t* p, const uint8_t (&c)[E]) {
  if constexpr (E == 2) *(uint16_t*)p = (uint16_t)(c[0] | (c[1] << 8));
  else p[0] = c[0];
}

// ---- int8, one scale per (token, kv head) -------------------------------------------------
// unit = (run, kv head, K|V): the consecutive tokens of the call that fall into one 16-token
// sub-block with consecutive slots.

// One run of `run` tokens starting at token t0, slot0 (any length, any start inside the
// sub-block): a lane owns D/64 channels of every token.
template <int D>
__device__ inline void int8_run(const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                                uint8_t* __restrict__ cache, float* __restrict__ scales, int H,
                                int bs, int kv, int h, int t0, int64_t slot0, int run, int lane) {
  constexpr int E = D / 64;  // channels per lane
  const int64_t blk = slot0 >> __builtin_ctz(bs);  // block sizes are powers of two
  const int off0 = (int)(slot0 - blk * bs);
  const int so = off0 & 15;  // position inside the sub-block
  uint8_t* tile = cache + tile_offset(blk, kv, h, H, bs, D);
  float* srow = scales + (((size_t)blk * 2 + kv) * H + h) * bs + off0;
  const uint16_t* src = (kv ? v : k) + ((size_t)t0 * H + h) * D + lane * E;
  const size_t tstride = (size_t)H * D;
  RowImage img[E];
  for (int i = 0; i < run; ++i) {
    uint32_t bits[E];
    uint32_t amax = 0;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      bits[e] = src[i * tstride + e];
      const uint32_t a = bits[e] & 0x7FFF;
      amax = a > amax ? a : amax;
    }
    amax = wave_max_u32(amax);  // |bf16| orders like its bit pattern
    const float s = (amax == 0) ? 0.0f : (float)((double)bf16_bits_to_float(amax) / 127.0);
    uint8_t c[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const uint8_t code = (amax == 0) ? (uint8_t)0 : int8_code(bf16_bits_to_float(bits[e]), s);
      c[e] = stored_byte(code, KVQ_INT8_TOKEN_HEAD);
    }
    if (kv == 0) {
      store_k<E>(tile + k_elem(off0 + i, lane * E, bs, D), c);
    } else {
#pragma unroll
      for (int e = 0; e < E; ++e) img[e].put(so + i, c[e]);
    }
    if (lane == 0) srow[i] = s;
  }
  if (kv == 1) {
#pragma unroll
    for (int e = 0; e < E; ++e)
      store_v_row(tile + v_elem(off0 - so, lane * E + e, bs, D), img[e], so, run);
  }
}

// The wavefront of a run's first token does the work (one token per sequence in a decode
// step: every wavefront has a run of its own and they all proceed in parallel).
template <int D>
__global__ __launch_bounds__(kWaves * 64) void write_int8_kernel(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int64_t* __restrict__ slot_mapping, int32_t num_tokens, uint8_t* __restrict__ cache,
    float* __restrict__ scales, int32_t H, int32_t bs) {
  const int lane = threadIdx.x & 63;
  const int64_t unit = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
  if (unit >= (int64_t)num_tokens * H * 2) return;
  const int kv = (int)(unit & 1);
  const int h = (int)((unit >> 1) % H);
  const int t0 = (int)((unit >> 1) / H);
  const int64_t slot0 = slot_mapping[t0];
  if (slot0 < 0) return;
  const int so = (int)(slot0 & 15);
  if (t0 > 0 && so > 0 && slot_mapping[t0 - 1] == slot0 - 1) return;  // not a run's first token
  int run = 1;
  while (run < 16 - so && t0 + run < num_tokens && slot_mapping[t0 + run] == slot0 + run) ++run;
  int8_run<D>(k, v, cache, scales, H, bs, kv, h, t0, slot0, run, lane);
}

// ---- int8, many tokens per call (prefill) --------------------------------------------------
// A run that fills a whole 16-token sub-block, the common case when a prompt is written at
// once, is handled with 16-byte loads: a lane owns 8 adjacent channels of 16 / G tokens
// (G = 512 / D groups of D / 8 lanes).  Which tokens depends on the cache order the codes go
// into: for K the tokens i * G + g (lane group g, load i), so that each store instruction of
// the wavefront fills whole quads; for V the tokens g * (16 / G) + i, so that the lane's bytes
// of one channel are adjacent in that channel's 16-token row.
//
// Rounding x / s: the fp32 product x * rcp(s) is within 2.3e-5 of the exact quotient
// (|quotient| <= 127, rcp within one ulp, one rounding for the product), so unless it lies
// within 4e-5 of a half-integer its nearest integer is the exact quotient's; the rare
// elements that do are decided in fp64 like everywhere else.  The scale is one correctly
// rounded fp32 division, which equals the fp64 quotient rounded once for every bf16 absmax.

template <int D>
__device__ inline void int8_subblock(const uint16_t* __restrict__ src, size_t tstride,
                                     uint8_t* __restrict__ tile, float* __restrict__ srow,
                                     int kv, int off0, int bs, int lane) {
  constexpr int CL = D / 8;    // lanes per token row
  constexpr int G = 64 / CL;   // lane groups = token rows per load instruction
  constexpr int NI = 16 / G;   // token rows per lane
  const int c = lane & (CL - 1), g = lane / CL;
  uint4 raw[NI];
  int tok[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    tok[i] = kv ? g * NI + i : i * G + g;
    raw[i] = *(const uint4*)(src + (size_t)tok[i] * tstride + 8 * c);
  }
  uint32_t vcode[8] = {0, 0, 0, 0, 0, 0, 0, 0};  // V: per channel, this lane's tokens' bytes
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const uint32_t w[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
    uint32_t amax = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t lo = w[j] & 0x7FFFu, hi = (w[j] >> 16) & 0x7FFFu;
      amax = amax > lo ? amax : lo;
      amax = amax > hi ? amax : hi;
    }
    amax = row_max_u32<CL>(amax);
    const float s = int8_scale(amax);
    const bool fast = s > 1e-30f;  // rcp of a denormal is not usable
    const float inv = fast ? __builtin_amdgcn_rcpf(s) : 0.0f;
    uint32_t kcode[2] = {0, 0};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float x = (e & 1) ? __uint_as_float(w[e >> 1] & 0xFFFF0000u)
                              : __uint_as_float(w[e >> 1] << 16);
      const float stored = int8_code_f32(x, s, inv, fast) + 128.0f;  // offset-binary, exact
      if (kv == 0) kcode[e >> 2] = __builtin_amdgcn_cvt_pk_u8_f32(stored, e & 3, kcode[e >> 2]);
      else vcode[e] = __builtin_amdgcn_cvt_pk_u8_f32(stored, i, vcode[e]);
    }
    if (kv == 0)
      *(uint2*)(tile + k_elem(off0 + tok[i], 8 * c, bs, D)) = make_uint2(kcode[0], kcode[1]);
    if (c == 0) srow[tok[i]] = s;
  }
  if (kv == 1) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      uint8_t* row = tile + v_elem(off0, 8 * c + e, bs, D) + g * NI;
      if constexpr (NI == 4) *(uint32_t*)row = vcode[e];
      else *(uint16_t*)row = (uint16_t)vcode[e];
    }
  }
}

// unit = (window of 16 consecutive tokens of the call, kv head, K|V): the wavefront handles
// every run that starts inside its window, so no wavefront is launched only to find that its
// token is not a run's first.
template <int D>
__global__ __launch_bounds__(kWaves * 64) void write_int8_bulk_kernel(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int64_t* __restrict__ slot_mapping, int32_t num_tokens, uint8_t* __restrict__ cache,
    float* __restrict__ scales, int32_t H, int32_t bs) {
  const int lane = threadIdx.x & 63;
  const int64_t unit = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
  const int windows = (num_tokens + 15) >> 4;
  if (unit >= (int64_t)windows * H * 2) return;
  const int kv = (int)(unit & 1);
  const int h = (int)((unit >> 1) % H);
  const int w0 = (int)((unit >> 1) / H) * 16;
  // lanes 0..15: is token w0 + lane the first of a run
  bool first = false;
  {
    const int t = w0 + lane;
    if (lane < 16 && t < num_tokens) {
      const int64_t slot = slot_mapping[t];
      if (slot >= 0) {
        const int so = (int)(slot & 15);
        first = !(t > 0 && so > 0 && slot_mapping[t - 1] == slot - 1);
      }
    }
  }
  uint32_t starts = (uint32_t)__ballot(first);
  const size_t tstride = (size_t)H * D;
  while (starts) {
    const int t0 = w0 + __builtin_ctz(starts);
    starts &= starts - 1;
    const int64_t slot0 = slot_mapping[t0];
    const int so = (int)(slot0 & 15);
    // lanes 0..15: does token t0 + lane continue the run
    const bool cont = lane < 16 - so && t0 + lane < num_tokens && slot_mapping[t0 + lane] == slot0 + lane;
    const uint32_t m = (uint32_t)__ballot(cont);
    const int run = __builtin_ctz(~m);  // lane 0 always continues
    if (run == 16) {
      const int64_t blk = slot0 >> __builtin_ctz(bs);  // block sizes are powers of two
      const int off0 = (int)(slot0 - blk * bs);
      int8_subblock<D>((kv ? v : k) + ((size_t)t0 * H + h) * D, tstride,
                       cache + tile_offset(blk, kv, h, H, bs, D),
                       scales + (((size_t)blk * 2 + kv) * H + h) * bs + off0, kv, off0, bs, lane);
    } else {
      int8_run<D>(k, v, cache, scales, H, bs, kv, h, t0, slot0, run, lane);
    }
  }
}

// ---- fp8-e4m3, one scale per (block, kv head) ---------------------------------------------
// unit = (run, kv head, K|V): the consecutive tokens of the call that fall into one block.

// One run of `run` tokens starting at token t0, slot0 (any length, any start inside the block,
// earlier codes re-expressed if the scale grows): a lane owns D/64 channels of every token.
template <int D>
__device__ inline void fp8_run(const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                               uint8_t* __restrict__ cache, float* __restrict__ scales, int H,
                               int bs, int kv, int h, int t0, int64_t slot0, int run, int lane,
                               bool tensor_scale) {
  constexpr int E = D / 64;
  const int64_t blk = slot0 >> __builtin_ctz(bs);  // block sizes are powers of two
  const int o_min = (int)(slot0 - blk * bs);
  const uint16_t* src = (kv ? v : k) + ((size_t)t0 * H + h) * D + lane * E;
  const size_t tstride = (size_t)H * D;
  // tensor_scale: the scale is the caller's (one per layer for K, one for V) and only read;
  // otherwise it is the block's, grown to cover this run
  uint32_t amax = 0;
  if (!tensor_scale) {
    for (int i = 0; i < run; ++i) {
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const uint32_t a = src[i * tstride + e] & 0x7FFF;
        amax = a > amax ? a : amax;
      }
    }
    amax = wave_max_u32(amax);
  }
  float* sp = tensor_scale ? scales + kv : scales + ((size_t)blk * 2 + kv) * H + h;
  const float s_prev = (tensor_scale || o_min > 0) ? *sp : 0.0f;
  const float s_cand = (amax == 0) ? 0.0f : (float)((double)bf16_bits_to_float(amax) / 448.0);
  const float s_new = s_prev > s_cand ? s_prev : s_cand;
  // the block's scale grew: the codes stored below the run are re-expressed in the new scale
  const bool regrade = o_min > 0 && s_new > s_prev && s_prev > 0.0f;
  auto regraded = [&](uint32_t c) -> uint8_t {
    if ((c & 0x7F) == 0x7F) return (uint8_t)c;  // NaN codes stay
    return fp8_code(fp8_value(c) * (double)s_prev / (double)s_new);
  };
  auto encoded = [&](int i, int e) -> uint8_t {
    if (!(s_new > 0.0f)) return 0;
    return fp8_code((double)bf16_bits_to_float(src[i * tstride + e]) / (double)s_new);
  };

  uint8_t* tile = cache + tile_offset(blk, kv, h, H, bs, D);
  if (kv == 0) {
    if (regrade) {
      for (int off = 0; off < o_min; ++off) {
        uint8_t* pc = tile + k_elem(off, lane * E, bs, D);
        uint8_t c[E];
#pragma unroll
        for (int e = 0; e < E; ++e) c[e] = regraded(pc[e]);
        store_k<E>(pc, c);
      }
    }
    for (int i = 0; i < run; ++i) {
      uint8_t c[E];
#pragma unroll
      for (int e = 0; e < E; ++e) c[e] = encoded(i, e);
      store_k<E>(tile + k_elem(o_min + i, lane * E, bs, D), c);
    }
  } else {
    // V: sub-block by sub-block, each channel's 16-token row read (if it holds older codes),
    // updated and stored once
    const int first_sb = regrade ? 0 : (o_min >> 4);
    const int last_sb = (o_min + run - 1) >> 4;
    for (int sb = first_sb; sb <= last_sb; ++sb) {
      const int lo = max(o_min - 16 * sb, 0);             // first new position in this row
      const int hi = min(o_min + run - 16 * sb, 16);      // one past the last new position
      const int old_n = regrade ? min(lo, 16) : 0;        // older codes to re-express: [0, old_n)
#pragma unroll
      for (int e = 0; e < E; ++e) {
        uint8_t* row = tile + v_elem(16 * sb, lane * E + e, bs, D);
        RowImage img;
        for (int j = 0; j < old_n; ++j) img.put(j, regraded(row[j]));
        for (int j = max(lo, 0); j < hi; ++j) img.put(j, encoded(16 * sb + j - o_min, e));
        const int first = old_n > 0 ? 0 : lo;  // older codes, if re-expressed, end where the new begin
        if (hi > first) store_v_row(row, img, first, hi - first);
      }
    }
  }
  if (lane == 0 && !tensor_scale) *sp = s_new;
}

template <int D>
__global__ __launch_bounds__(kWaves * 64) void write_fp8_kernel(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int64_t* __restrict__ slot_mapping, int32_t num_tokens, uint8_t* __restrict__ cache,
    float* __restrict__ scales, int32_t H, int32_t bs, int32_t tensor_scale) {
  const int lane = threadIdx.x & 63;
  const int64_t unit = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
  if (unit >= (int64_t)num_tokens * H * 2) return;
  const int kv = (int)(unit & 1);
  const int h = (int)((unit >> 1) % H);
  const int t0 = (int)((unit >> 1) / H);
  const int64_t slot0 = slot_mapping[t0];
  if (slot0 < 0) return;
  const int o_min = (int)(slot0 & (bs - 1));
  if (t0 > 0 && o_min > 0 && slot_mapping[t0 - 1] == slot0 - 1) return;  // not a run's first token
  int run = 1;
  while (run < bs - o_min && t0 + run < num_tokens && slot_mapping[t0 + run] == slot0 + run) ++run;
  fp8_run<D>(k, v, cache, scales, H, bs, kv, h, t0, slot0, run, lane, tensor_scale != 0);
}

// ---- fp8, many tokens per call (prefill) ---------------------------------------------------
// A run made of whole 16-token sub-blocks whose block scale does not force a re-encode of
// earlier codes (always so when a block is written at once) is handled with 16-byte loads, a
// lane owning 8 channels of 16 / G tokens as in the int8 prefill kernel: one pass for the
// run's absmax, a second (the rows now come from the cache) for the codes.
//
// Rounding x / s to E4M3: with q = x * rcp(s) in fp32 (relative error below 1.8e-7) and
// t = |q| / 2^(e-3), e = max(floor(log2 |q|), -6), the code's mantissa is the nearest integer
// to t in [0, 16]; t is within 3e-6 of the exact value, so unless it lies within 1e-5 of a
// half-integer its nearest integer is the exact one's.  (Just below a power of two the fast
// exponent may come out one higher than the exact one; t is then 8 and the code the same.)
// The rare elements near a half-integer are decided in fp64.
__device__ inline uint32_t fp8_code_fast(float x, float inv, float s, bool usable) {
  const float q = x * inv;
  const float a = fminf(fabsf(q), 448.0f);
  int e = (int)(__float_as_uint(a) >> 23) - 127;
  e = e < -6 ? -6 : e;
  const float t = __builtin_ldexpf(a, 3 - e);
  const float r = __builtin_rintf(t);
  if (__builtin_expect(!usable || fabsf(t - r) > 0.5f - 1e-5f, 0))
    return fp8_code((double)x / (double)s);
  return ((__float_as_uint(q) >> 24) & 0x80u) | (uint32_t)(((e + 7) << 3) + (int)r - 8);
}

template <int D>
__device__ inline void fp8_subblocks(const uint16_t* __restrict__ src, size_t tstride,
                                     uint8_t* __restrict__ tile, float* __restrict__ sp, int kv,
                                     int o_min, int run, int bs, int lane, bool tensor_scale,
                                     bool& done) {
  constexpr int CL = D / 8, G = 64 / CL, NI = 16 / G;
  const int c = lane & (CL - 1), g = lane / CL;
  int tok[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) tok[i] = kv ? g * NI + i : i * G + g;
  uint32_t amax = 0;
  if (!tensor_scale) {
    for (int sb = 0; sb < run; sb += 16) {
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        const uint4 raw = *(const uint4*)(src + (size_t)(sb + tok[i]) * tstride + 8 * c);
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t lo = w[j] & 0x7FFFu, hi = (w[j] >> 16) & 0x7FFFu;
          amax = amax > lo ? amax : lo;
          amax = amax > hi ? amax : hi;
        }
      }
    }
    amax = wave_max_u32(amax);
  }
  const float s_prev = (tensor_scale || o_min > 0) ? *sp : 0.0f;
  const float s_cand = (amax == 0) ? 0.0f : __fdiv_rn(bf16_bits_to_float(amax), 448.0f);
  const float s_new = s_prev > s_cand ? s_prev : s_cand;
  done = !(o_min > 0 && s_new > s_prev && s_prev > 0.0f);
  if (!done) return;  // earlier codes must be re-expressed: the general routine does the run
  const bool usable = s_new > 1e-30f;  // rcp of a denormal is not usable
  const float inv = usable ? __builtin_amdgcn_rcpf(s_new) : 0.0f;
  for (int sb = 0; sb < run; sb += 16) {
    uint32_t vcode[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const uint4 raw = *(const uint4*)(src + (size_t)(sb + tok[i]) * tstride + 8 * c);
      const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
      uint32_t kcode[2] = {0, 0};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float x = (e & 1) ? __uint_as_float(w[e >> 1] & 0xFFFF0000u)
                                : __uint_as_float(w[e >> 1] << 16);
        const uint32_t code = (s_new > 0.0f) ? fp8_code_fast(x, inv, s_new, usable) : 0u;
        if (kv == 0) kcode[e >> 2] |= code << (8 * (e & 3));
        else vcode[e] |= code << (8 * i);
      }
      if (kv == 0)
        *(uint2*)(tile + k_elem(o_min + sb + tok[i], 8 * c, bs, D)) = make_uint2(kcode[0], kcode[1]);
    }
    if (kv == 1) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        uint8_t* row = tile + v_elem(o_min + sb, 8 * c + e, bs, D) + g * NI;
        if constexpr (NI == 4) *(uint32_t*)row = vcode[e];
        else *(uint16_t*)row = (uint16_t)vcode[e];
      }
    }
  }
  if (lane == 0 && !tensor_scale) *sp = s_new;
}

// unit = (window of 16 consecutive tokens of the call, kv head, K|V), as for int8
template <int D>
__global__ __launch_bounds__(kWaves * 64) void write_fp8_bulk_kernel(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int64_t* __restrict__ slot_mapping, int32_t num_tokens, uint8_t* __restrict__ cache,
    float* __restrict__ scales, int32_t H, int32_t bs, int32_t tensor_scale) {
  const int lane = threadIdx.x & 63;
  const int64_t unit = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
  const int windows = (num_tokens + 15) >> 4;
  if (unit >= (int64_t)windows * H * 2) return;
  const int kv = (int)(unit & 1);
  const int h = (int)((unit >> 1) % H);
  const int w0 = (int)((unit >> 1) / H) * 16;
  bool first = false;
  {
    const int t = w0 + lane;
    if (lane < 16 && t < num_tokens) {
      const int64_t slot = slot_mapping[t];
      if (slot >= 0)
        first = !(t > 0 && (slot & (bs - 1)) > 0 && slot_mapping[t - 1] == slot - 1);
    }
  }
  uint32_t starts = (uint32_t)__ballot(first);
  const size_t tstride = (size_t)H * D;
  while (starts) {
    const int t0 = w0 + __builtin_ctz(starts);
    starts &= starts - 1;
    const int64_t slot0 = slot_mapping[t0];
    const int o_min = (int)(slot0 & (bs - 1));
    int run = 0;
    for (int base = 0; base < bs - o_min; base += 64) {  // block sizes reach 256
      const int j = base + lane;
      const bool cont = j < bs - o_min && t0 + j < num_tokens && slot_mapping[t0 + j] == slot0 + j;
      const unsigned long long m = __ballot(cont);
      const int n = m == ~0ull ? 64 : __builtin_ctzll(~m);
      run += n;
      if (n < 64) break;
    }
    bool done = false;
    if (((o_min | run) & 15) == 0) {
      const int64_t blk = slot0 >> __builtin_ctz(bs);
      fp8_subblocks<D>((kv ? v : k) + ((size_t)t0 * H + h) * D, tstride,
                       cache + tile_offset(blk, kv, h, H, bs, D),
                       tensor_scale ? scales + kv : scales + ((size_t)blk * 2 + kv) * H + h, kv,
                       o_min, run, bs, lane, tensor_scale != 0, done);
    }
    if (!done)
      fp8_run<D>(k, v, cache, scales, H, bs, kv, h, t0, slot0, run, lane, tensor_scale != 0);
  }
}

// ---- int4, one scale per (token, kv head), head_dim 128 ------------------------------------
// As int8 with 7 in place of 127 and two codes per byte; a code is stored as the nibble
// code + 8.  The 32-bit word / nibble a logical element lives in is given by int4_k_word,
// int4_v_word and int4_nibble.
__device__ inline uint32_t int4_nib(float x, float s) {  // stored nibble of x / s, exact rounding
  double r = rint((double)x / (double)s);
  r = r > 7.0 ? 7.0 : r;
  r = r < -7.0 ? -7.0 : r;
  return (uint32_t)((int)r + 8);
}

// One run (consecutive tokens with consecutive slots inside one 16-token sub-block).  A lane
// owns channels 2 lane and 2 lane + 1.  K: the four lanes of a quad hold the eight codes of one
// word and combine them with two cross-lane ORs.  V: the lane owns its two channels' 16-token
// rows (8 bytes each): a run that fills the sub-block stores them whole; a shorter run clears and
// sets only its own nibbles with integer atomics on the two 32-bit words, because other runs of
// the same call (a skipped token in mid sub-block, tokens not in slot order) are handled by
// other wavefronts and share those words.  The nibbles of different tokens are disjoint, so the
// result does not depend on the order in which the wavefronts arrive.
__device__ inline void int4_run(const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                                uint8_t* __restrict__ cache, float* __restrict__ scales, int H,
                                int bs, int kv, int h, int t0, int64_t slot0, int run, int lane) {
  constexpr int D = 128;
  const int64_t blk = slot0 >> __builtin_ctz(bs);
  const int off0 = (int)(slot0 - blk * bs);
  const int so = off0 & 15;
  uint8_t* tile = cache + (size_t)tile_offset(blk, kv, h, H, bs, D / 2);
  float* srow = scales + (((size_t)blk * 2 + kv) * H + h) * bs + off0;
  const uint16_t* src = (kv ? v : k) + ((size_t)t0 * H + h) * D + lane * 2;
  const size_t tstride = (size_t)H * D;
  unsigned long long img[2] = {0, 0}, mask = 0;  // V rows of the lane's two channels
  for (int i = 0; i < run; ++i) {
    const uint32_t w = *(const uint32_t*)(src + i * tstride);
    const uint32_t b0 = w & 0xFFFFu, b1 = w >> 16;
    uint32_t amax = (b0 & 0x7FFFu) > (b1 & 0x7FFFu) ? (b0 & 0x7FFFu) : (b1 & 0x7FFFu);
    amax = wave_max_u32(amax);
    const float s = (amax == 0) ? 0.0f : (float)((double)bf16_bits_to_float(amax) / 7.0);
    const uint32_t n0 = (amax == 0) ? 8u : int4_nib(bf16_bits_to_float(b0), s);
    const uint32_t n1 = (amax == 0) ? 8u : int4_nib(bf16_bits_to_float(b1), s);
    if (kv == 0) {
      // channels 2 lane, 2 lane + 1 are elements 2 (lane % 4) and + 1 of their word
      uint32_t word = (n0 << (4 * (lane & 3))) | (n1 << (4 * ((lane & 3) + 4)));
      word |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)word, 0xB1, 0xF, 0xF, false);
      word |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)word, 0x4E, 0xF, 0xF, false);
      if ((lane & 3) == 0) *(uint32_t*)(tile + int4_k_word(off0 + i, 2 * lane)) = word;
    } else {
      const int t = so + i;  // position in the sub-block: word t / 8, element t % 8
      const int sh = 32 * (t >> 3) + 4 * int4_nibble(t & 7);
      img[0] |= (unsigned long long)n0 << sh;
      img[1] |= (unsigned long long)n1 << sh;
      mask |= 15ull << sh;
    }
    if (lane == 0) srow[i] = s;
  }
  if (kv == 1) {
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      uint8_t* row = tile + int4_v_word(off0 - so, 2 * lane + e);
      if (run == 16) {
        *(unsigned long long*)row = img[e];
      } else {
#pragma unroll
        for (int wd = 0; wd < 2; ++wd) {  // tokens 0-7 and 8-15 of the sub-block
          const uint32_t mw = (uint32_t)(mask >> (32 * wd));
          if (mw == 0) continue;
          uint32_t* word = (uint32_t*)row + wd;
          atomicAnd(word, ~mw);
          atomicOr(word, (uint32_t)(img[e] >> (32 * wd)));
        }
      }
    }
  }
}

__global__ __launch_bounds__(kWaves * 64) void write_int4_kernel(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int64_t* __restrict__ slot_mapping, int32_t num_tokens, uint8_t* __restrict__ cache,
    float* __restrict__ scales, int32_t H, int32_t bs) {
  const int lane = threadIdx.x & 63;
  const int64_t unit = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
  if (unit >= (int64_t)num_tokens * H * 2) return;
  const int kv = (int)(unit & 1);
  const int h = (int)((unit >> 1) % H);
  const int t0 = (int)((unit >> 1) / H);
  const int64_t slot0 = slot_mapping[t0];
  if (slot0 < 0) return;
  const int so = (int)(slot0 & 15);
  if (t0 > 0 && so > 0 && slot_mapping[t0 - 1] == slot0 - 1) return;  // not a run's first token
  int run = 1;
  while (run < 16 - so && t0 + run < num_tokens && slot_mapping[t0 + run] == slot0 + run) ++run;
  int4_run(k, v, cache, scales, H, bs, kv, h, t0, slot0, run, lane);
}

// A whole sub-block with 16-byte loads, as for int8: a lane owns 8 channels (8 c .. 8 c + 7,
// c = lane % 16) of 4 tokens.  K (tokens 4 i + g): the lane's eight codes of a token are one
// whole word.  V (tokens 4 g + i): the lane's four tokens of a channel are the nibbles
// 2a, 2a+1 (one byte) and 2a+4, 2a+5 (another byte) of the channel's word g / 2, a = g % 2.
__device__ inline void int4_subblock(const uint16_t* __restrict__ src, size_t tstride,
                                     uint8_t* __restrict__ tile, float* __restrict__ srow,
                                     int kv, int off0, int lane) {
  const int c = lane & 15, g = lane >> 4;
  uint4 raw[4];
  int tok[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    tok[i] = kv ? g * 4 + i : i * 4 + g;
    raw[i] = *(const uint4*)(src + (size_t)tok[i] * tstride + 8 * c);
  }
  uint32_t vnib[8][4];  // V: [channel][token i]
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t w[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
    uint32_t amax = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t lo = w[j] & 0x7FFFu, hi = (w[j] >> 16) & 0x7FFFu;
      amax = amax > lo ? amax : lo;
      amax = amax > hi ? amax : hi;
    }
    amax = row_max_u32<16>(amax);
    const float a = bf16_bits_to_float(amax);
    const float s = (amax == 0) ? 0.0f : __fdiv_rn(a, 7.0f);
    const bool fast = s > 1e-30f;
    const float inv = fast ? __builtin_amdgcn_rcpf(s) : 0.0f;
    uint32_t kword = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float x = (e & 1) ? __uint_as_float(w[e >> 1] & 0xFFFF0000u)
                              : __uint_as_float(w[e >> 1] << 16);
      const float q = x * inv;
      const float r = __builtin_rintf(q);
      uint32_t nib = (uint32_t)((int)r + 8);
      if (__builtin_expect(!fast || fabsf(q - r) > 0.5f - 4e-5f, 0))
        nib = (amax == 0) ? 8u : int4_nib(x, s);
      if (kv == 0) kword |= nib << (4 * int4_nibble(e));
      else vnib[e][i] = nib;
    }
    if (kv == 0) *(uint32_t*)(tile + int4_k_word(off0 + tok[i], 8 * c)) = kword;
    if (c == 0) srow[tok[i]] = s;
  }
  if (kv == 1) {
    const int a = g & 1;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      uint8_t* word = tile + int4_v_word(off0 + 8 * (g >> 1), 8 * c + e);
      word[a] = (uint8_t)(vnib[e][0] | (vnib[e][2] << 4));      // elements 4a, 4a+2
      word[a + 2] = (uint8_t)(vnib[e][1] | (vnib[e][3] << 4));  // elements 4a+1, 4a+3
    }
  }
}

__global__ __launch_bounds__(kWaves * 64) void write_int4_bulk_kernel(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int64_t* __restrict__ slot_mapping, int32_t num_tokens, uint8_t* __restrict__ cache,
    float* __restrict__ scales, int32_t H, int32_t bs) {
  constexpr int D = 128;
  const int lane = threadIdx.x & 63;
  const int64_t unit = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
  const int windows = (num_tokens + 15) >> 4;
  if (unit >= (int64_t)windows * H * 2) return;
  const int kv = (int)(unit & 1);
  const int h = (int)((unit >> 1) % H);
  const int w0 = (int)((unit >> 1) / H) * 16;
  bool first = false;
  {
    const int t = w0 + lane;
    if (lane < 16 && t < num_tokens) {
      const int64_t slot = slot_mapping[t];
      if (slot >= 0) first = !(t > 0 && (slot & 15) > 0 && slot_mapping[t - 1] == slot - 1);
    }
  }
  uint32_t starts = (uint32_t)__ballot(first);
  const size_t tstride = (size_t)H * D;
  while (starts) {
    const int t0 = w0 + __builtin_ctz(starts);
    starts &= starts - 1;
    const int64_t slot0 = slot_mapping[t0];
    const int so = (int)(slot0 & 15);
    const bool cont = lane < 16 - so && t0 + lane < num_tokens && slot_mapping[t0 + lane] == slot0 + lane;
    const int run = __builtin_ctz(~(uint32_t)__ballot(cont));
    if (run == 16) {
      const int64_t blk = slot0 >> __builtin_ctz(bs);
      const int off0 = (int)(slot0 - blk * bs);
      int4_subblock((kv ? v : k) + ((size_t)t0 * H + h) * D, tstride,
                    cache + (size_t)tile_offset(blk, kv, h, H, bs, D / 2),
                    scales + (((size_t)blk * 2 + kv) * H + h) * bs + off0, kv, off0, lane);
    } else {
      int4_run(k, v, cache, scales, H, bs, kv, h, t0, slot0, run, lane);
    }
  }
}

// ---- unquantized cache: the rows are copied to their slots ---------------------------------
// unit = (token, kv head, K|V); a lane moves D/64 adjacent channels.
template <int D>
__global__ __launch_bounds__(kWaves * 64) void write_plain_kernel(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int64_t* __restrict__ slot_mapping, int32_t num_tokens, uint16_t* __restrict__ cache,
    int32_t H, int32_t bs) {
  constexpr int E = D / 64;
  const int lane = threadIdx.x & 63;
  const int64_t unit = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
  if (unit >= (int64_t)num_tokens * H * 2) return;
  const int kv = (int)(unit & 1);
  const int h = (int)((unit >> 1) % H);
  const int t = (int)((unit >> 1) / H);
  const int64_t slot = slot_mapping[t];
  if (slot < 0) return;
  const int64_t blk = slot >> __builtin_ctz(bs);
  const int off = (int)(slot & (bs - 1));
  const uint16_t* src = (kv ? v : k) + ((size_t)t * H + h) * D + lane * E;
  uint16_t* tile = cache + tile_offset(blk, kv, h, H, bs, D);  // in elements
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int d = lane * E + e;
    tile[kv ? v_elem16(off, d, D) : k_elem16(off, d, D)] = src[e];
  }
}

}  // namespace

hipError_t launch_write(const void* k, const void* v, const int64_t* slot_mapping,
                        int32_t num_tokens, void* cache, float* scales,
                        const kvq_cache_desc_t& desc, hipStream_t stream) {
  // many tokens (a prompt): a wavefront per window of 16 tokens; few (a decode step): a
  // wavefront per token, so that runs are handled in parallel rather than one after another
  const bool bulk = num_tokens >= kBulkTokens;
  const int64_t units =
      (int64_t)(bulk ? (num_tokens + 15) / 16 : num_tokens) * desc.num_kv_heads * 2;
  const unsigned grid = (unsigned)((units + kWaves - 1) / kWaves);
  const dim3 block(kWaves * 64);
  const uint16_t* kk = (const uint16_t*)k;
  const uint16_t* vv = (const uint16_t*)v;
  uint8_t* c = (uint8_t*)cache;
#define KVQ_LAUNCH_WRITE(KERNEL, DD)                                                          \
  hipLaunchKernelGGL((KERNEL<DD>), dim3(grid), block, 0, stream, kk, vv, slot_mapping,        \
                     num_tokens, c, scales, desc.num_kv_heads, desc.block_size)
#define KVQ_LAUNCH_WRITE_FP8(KERNEL, DD)                                                      \
  hipLaunchKernelGGL((KERNEL<DD>), dim3(grid), block, 0, stream, kk, vv, slot_mapping,        \
                     num_tokens, c, scales, desc.num_kv_heads, desc.block_size,               \
                     (int32_t)(desc.mode == KVQ_FP8E4M3_TENSOR))
  if (desc.mode == KVQ_INT4_TOKEN_HEAD) {
    if (bulk)
      hipLaunchKernelGGL(write_int4_bulk_kernel, dim3(grid), block, 0, stream, kk, vv, slot_mapping,
                         num_tokens, c, scales, desc.num_kv_heads, desc.block_size);
    else
      hipLaunchKernelGGL(write_int4_kernel, dim3(grid), block, 0, stream, kk, vv, slot_mapping,
                         num_tokens, c, scales, desc.num_kv_heads, desc.block_size);
  } else if (desc.mode == KVQ_BF16_PLAIN) {
    const unsigned g = (unsigned)(((int64_t)num_tokens * desc.num_kv_heads * 2 + kWaves - 1) / kWaves);
    if (desc.head_dim == 128)
      hipLaunchKernelGGL((write_plain_kernel<128>), dim3(g), block, 0, stream, kk, vv, slot_mapping,
                         num_tokens, (uint16_t*)cache, desc.num_kv_heads, desc.block_size);
    else
      hipLaunchKernelGGL((write_plain_kernel<64>), dim3(g), block, 0, stream, kk, vv, slot_mapping,
                         num_tokens, (uint16_t*)cache, desc.num_kv_heads, desc.block_size);
  } else if (bulk && desc.mode == KVQ_INT8_TOKEN_HEAD) {
    if (desc.head_dim == 128) KVQ_LAUNCH_WRITE(write_int8_bulk_kernel, 128);
    else KVQ_LAUNCH_WRITE(write_int8_bulk_kernel, 64);
  } else if (bulk) {
    if (desc.head_dim == 128) KVQ_LAUNCH_WRITE_FP8(write_fp8_bulk_kernel, 128);
    else KVQ_LAUNCH_WRITE_FP8(write_fp8_bulk_kernel, 64);
  } else if (desc.mode == KVQ_INT8_TOKEN_HEAD) {
    if (desc.head_dim == 128) KVQ_LAUNCH_WRITE(write_int8_kernel, 128);
    else KVQ_LAUNCH_WRITE(write_int8_kernel, 64);
  } else {
    if (desc.head_dim == 128) KVQ_LAUNCH_WRITE_FP8(write_fp8_kernel, 128);
    else KVQ_LAUNCH_WRITE_FP8(write_fp8_kernel, 64);
  }
#undef KVQ_LAUNCH_WRITE
#undef KVQ_LAUNCH_WRITE_FP8
  return hipGetLastError();
}

}  // namespace kvq
