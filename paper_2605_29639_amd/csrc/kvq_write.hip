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
// Each format has a general routine (any run, one token after another) and one that takes a
// 16-token sub-block at a time, which calls carrying a prompt use (16-byte loads, fp32 rounding
// with an fp64 decision near ties; for int8 and fp8 a wavefront does K and V of its window and
// runs shorter than a sub-block go the same way with the missing rows masked).
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
// Rounding x / s without fp64 and without a branch per element: t = fma(x, rcp(s), 1.5 * 2^23 +
// 128) is the product rounded once to an integer (the unit in the last place up there is 1,
// ties go to even) plus 128, so the low byte of t's bit pattern is the stored code.  The
// product differs from the exact quotient by at most 1.6e-5 (|quotient| <= 127, rcp within one
// ulp), so t holds the exact quotient's rounding unless the quotient lies within that distance
// of a half-integer; d = fma(x, rcp(s), -(t - 1.5 * 2^23 - 128)) measures it, and the elements
// with |d| > 0.5 - 4e-5 (about one in 12 000), like rows whose scale is zero or below the normal
// fp32 range, are marked in a bit mask and decided in fp64 afterwards, the wavefront skipping
// every element nobody marked.  The scale is one correctly rounded fp32 division, which equals
// the fp64 quotient rounded once for every bf16 absmax.
constexpr float kRoundMagic = 12582912.0f + 128.0f;  // 1.5 * 2^23 + 128

typedef unsigned short ushort2v __attribute__((ext_vector_type(2)));

// largest |bf16| bit pattern among the 8 values of a 16-byte piece
__device__ inline uint32_t absmax8(const uint4& raw) {
  const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
  ushort2v m = {0, 0};
#pragma unroll
  for (int j = 0; j < 4; ++j)
    m = __builtin_elementwise_max(m, __builtin_bit_cast(ushort2v, w[j] & 0x7FFF7FFFu));
  return m[0] > m[1] ? m[0] : m[1];
}
__device__ inline float bf16_of(const uint4& raw, int e) {  // element e of the 8
  const uint32_t w = e < 2 ? raw.x : e < 4 ? raw.y : e < 6 ? raw.z : raw.w;
  return (e & 1) ? __uint_as_float(w & 0xFFFF0000u) : __uint_as_float(w << 16);
}
// the low bytes of four words, packed in order
__device__ inline uint32_t low_bytes(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  return __builtin_amdgcn_perm(b, a, 0x0c0c0400u) | __builtin_amdgcn_perm(d, c, 0x04000c0cu);
}

// The rows of a sub-block, 16 / G of them per lane (which ones depends on K or V, see above).
// Rows r_lo .. r_hi - 1 of the sub-block are the run's tokens (all 16 for a whole sub-block);
// `src` is where row r_lo's token lies; the other rows are not read.
template <int D>
__device__ inline void load_subblock(const uint16_t* __restrict__ src, size_t tstride, int kv,
                                     int lane, int r_lo, int r_hi, uint4 (&raw)[D / 32]) {
  constexpr int CL = D / 8, G = 64 / CL, NI = 16 / G;
  const int c = lane & (CL - 1), g = lane / CL;
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int r = kv ? g * NI + i : i * G + g;
    raw[i] = (r >= r_lo && r < r_hi) ? *(const uint4*)(src + (ptrdiff_t)(r - r_lo) * (ptrdiff_t)tstride + 8 * c)
                                     : make_uint4(0u, 0u, 0u, 0u);
  }
}

template <int D>
__device__ inline void int8_subblock(const uint4 (&raw)[D / 32], uint8_t* __restrict__ tile,
                                     float* __restrict__ srow, int kv, int off0, int bs, int lane,
                                     int r_lo, int r_hi) {
  constexpr int CL = D / 8;    // lanes per token row
  constexpr int G = 64 / CL;   // lane groups = token rows per load instruction
  constexpr int NI = 16 / G;   // token rows per lane
  const int c = lane & (CL - 1), g = lane / CL;
  int tok[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) tok[i] = kv ? g * NI + i : i * G + g;
  uint32_t vcode[8] = {0, 0, 0, 0, 0, 0, 0, 0};  // V: per channel, this lane's tokens' bytes
  float mine = 0.0f;  // the scale this lane stores
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const float s = int8_scale(row_max_u32<CL>(absmax8(raw[i])));
    const bool fast = s > 1e-30f;  // rcp of a denormal is not usable
    const float inv = fast ? __builtin_amdgcn_rcpf(s) : 0.0f;
    uint32_t t[8];  // bit patterns of 1.5 * 2^23 + 128 + code: the low byte is the stored code
    // lanes whose element e needs the exact decision (wave-wide masks: the comparisons write
    // them directly and the scalar unit collects them)
    unsigned long long marked[8], any_marked = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float x = bf16_of(raw[i], e);
      const float tf = __builtin_fmaf(x, inv, kRoundMagic);
      const float d = __builtin_fmaf(x, inv, -(tf - kRoundMagic));
      t[e] = __float_as_uint(tf);
      marked[e] = __ballot(!fast || fabsf(d) > 0.5f - 4e-5f);
      any_marked |= marked[e];
    }
    if (__builtin_expect(any_marked != 0, 0)) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (marked[e] == 0) continue;  // wave-uniform: nobody asked
        if ((marked[e] >> lane) & 1)
          t[e] = s == 0.0f ? 128u : (uint32_t)((int8_t)int8_code(bf16_of(raw[i], e), s) + 128);
      }
    }
    if (kv == 0) {
      if (tok[i] >= r_lo && tok[i] < r_hi)
        *(uint2*)(tile + k_elem(off0 + tok[i], 8 * c, bs, D)) =
            make_uint2(low_bytes(t[0], t[1], t[2], t[3]), low_bytes(t[4], t[5], t[6], t[7]));
    } else {
      // the low byte of t[e] becomes byte i of the channel's word
      constexpr uint32_t kInsert[4] = {0x03020104u, 0x03020400u, 0x03040100u, 0x04020100u};
#pragma unroll
      for (int e = 0; e < 8; ++e) vcode[e] = __builtin_amdgcn_perm(t[e], vcode[e], kInsert[i]);
    }
    mine = c == i ? s : mine;
  }
  // the sub-block's 16 scales in one store: lane (c = i, group g) writes its row i's
  if (c < NI) {
    const int r = kv ? g * NI + c : c * G + g;
    if (r >= r_lo && r < r_hi) srow[r] = mine;
  }
  if (kv == 1) {
    const bool whole = r_lo == 0 && r_hi == 16;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      uint8_t* row = tile + v_elem(off0, 8 * c + e, bs, D) + g * NI;
      if (whole) {
        if constexpr (NI == 4) *(uint32_t*)row = vcode[e];
        else *(uint16_t*)row = (uint16_t)vcode[e];
      } else {  // a shorter run: byte by byte, the other slots of the row keep their contents
#pragma unroll
        for (int i = 0; i < NI; ++i)
          if (g * NI + i >= r_lo && g * NI + i < r_hi) row[i] = (uint8_t)(vcode[e] >> (8 * i));
      }
    }
  }
}

// unit = (window of 16 consecutive tokens of the call, kv head): the wavefront handles every run
// that starts inside its window, so no wavefront is launched only to find that its token is
// not a run's first, and it handles K and V alike: the slots are worked out once, and the V
// rows of a whole sub-block are already on their way while the K rows are encoded.
template <int D>
__global__ __launch_bounds__(kWaves * 64) void write_int8_bulk_kernel(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int64_t* __restrict__ slot_mapping, int32_t num_tokens, uint8_t* __restrict__ cache,
    float* __restrict__ scales, int32_t H, int32_t bs) {
  const int lane = threadIdx.x & 63;
  const int64_t unit = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
  const int windows = (num_tokens + 15) >> 4;
  if (unit >= (int64_t)windows * H) return;
  const int h = (int)(unit % H);
  const int w0 = (int)(unit / H) * 16;
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
    // rows so .. so + run - 1 of the sub-block that starts at block offset off0
    const int64_t blk = slot0 >> __builtin_ctz(bs);  // block sizes are powers of two
    const int off0 = (int)(slot0 - blk * bs) - so;
    const size_t row0 = ((size_t)t0 * H + h) * D;
    uint4 k_rows[D / 32], v_rows[D / 32];
    load_subblock<D>(k + row0, tstride, 0, lane, so, so + run, k_rows);
    load_subblock<D>(v + row0, tstride, 1, lane, so, so + run, v_rows);
    int8_subblock<D>(k_rows, cache + tile_offset(blk, 0, h, H, bs, D),
                     scales + (((size_t)blk * 2 + 0) * H + h) * bs + off0, 0, off0, bs, lane, so,
                     so + run);
    int8_subblock<D>(v_rows, cache + tile_offset(blk, 1, h, H, bs, D),
                     scales + (((size_t)blk * 2 + 1) * H + h) * bs + off0, 1, off0, bs, lane, so,
                     so + run);
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
// lane owning 8 channels of 16 / G tokens as in the int8 prefill kernel.  The rows of the run's
// first sub-block stay in registers between the pass that finds the run's absmax and the pass
// that encodes (a 16-token block is read once); further sub-blocks are read a second time.
// (Blocks above 16 tokens go to write_fp8_block_kernel below, a wavefront per sub-block.)
//
// Rounding x / s to E4M3 with the hardware conversion (v_cvt_pk_fp8_f32: nearest, ties to even,
// exact for every |value| <= 448 including the subnormals and the sign of zero; above 464 it
// gives NaN, so values are first limited to +-448): q = x * rcp(s) is within 1.8e-7 (relative)
// of the exact quotient, and the conversion is monotonic, so if q (1 + 2^-21) and q (1 - 2^-21)
// convert to the same code, that is the exact quotient's code.  The rare elements where they
// differ (a code boundary lies in between: about one in 60 000), and runs whose scale is below
// the normal fp32 range, are decided in fp64.
// Rows r_lo .. r_hi - 1 of the 16-token sub-block at block offset `base`, held in `raw` in the
// order load_subblock leaves them, encoded under the scale s and stored into the K or V tile.
template <int D>
__device__ inline void fp8_encode_subblock(const uint4 (&raw)[16 / (64 / (D / 8))], int kv,
                                           uint8_t* __restrict__ tile, int base, int r_lo, int r_hi,
                                           float s, int bs, int lane) {
  constexpr int CL = D / 8, G = 64 / CL, NI = 16 / G;
  constexpr float kUp = 1.0f + 4.76837158203125e-07f, kDown = 1.0f - 4.76837158203125e-07f;  // 2^-21
  const int c = lane & (CL - 1), g = lane / CL;
  const bool usable = s > 1e-30f;  // rcp of a denormal is not usable
  const float inv = usable ? __builtin_amdgcn_rcpf(s) : 0.0f;
  // four values (element e4[n] of row r4[n]) -> four code bytes in that order
  auto codes4 = [&](const int (&r4)[4], const int (&e4)[4], int n) -> uint32_t {
    if (!(s > 0.0f)) return 0u;  // an all-zero run under a zero scale: codes 0x00
    float q[4];
#pragma unroll
    for (int x = 0; x < 4; ++x)
      q[x] = x < n ? __builtin_amdgcn_fmed3f(bf16_of(raw[r4[x]], e4[x]) * inv, -448.0f, 448.0f) : 0.0f;
    int up = __builtin_amdgcn_cvt_pk_fp8_f32(q[0] * kUp, q[1] * kUp, 0, false);
    int down = __builtin_amdgcn_cvt_pk_fp8_f32(q[0] * kDown, q[1] * kDown, 0, false);
    if (n > 2) {
      up = __builtin_amdgcn_cvt_pk_fp8_f32(q[2] * kUp, q[3] * kUp, up, true);
      down = __builtin_amdgcn_cvt_pk_fp8_f32(q[2] * kDown, q[3] * kDown, down, true);
    }
    uint32_t word = (uint32_t)up;
    const uint32_t diff = usable ? word ^ (uint32_t)down : ~0u;
    if (__builtin_expect(__any(diff != 0), 0)) {
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        if (x >= n) break;
        const bool bad = ((diff >> (8 * x)) & 0xFFu) != 0;
        if (!__any(bad)) continue;  // wave-uniform: nobody asked
        if (bad) {
          const uint32_t code = fp8_code((double)bf16_of(raw[r4[x]], e4[x]) / (double)s);
          word = (word & ~(0xFFu << (8 * x))) | (code << (8 * x));
        }
      }
    }
    return word;
  };
  if (kv == 0) {  // a row's 8 codes are two words of the quad order
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int r = i * G + g;
      const int r4[4] = {i, i, i, i}, lo[4] = {0, 1, 2, 3}, hi[4] = {4, 5, 6, 7};
      const uint2 words = make_uint2(codes4(r4, lo, 4), codes4(r4, hi, 4));
      if (r >= r_lo && r < r_hi) *(uint2*)(tile + k_elem(base + r, 8 * c, bs, D)) = words;
    }
  } else {  // a channel's NI tokens are adjacent bytes of its 16-token row
    const bool whole = r_lo == 0 && r_hi == 16;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int r4[4] = {0, 1 % NI, 2 % NI, 3 % NI}, e4[4] = {e, e, e, e};
      const uint32_t word = codes4(r4, e4, NI);
      uint8_t* row = tile + v_elem(base, 8 * c + e, bs, D) + g * NI;
      if (whole) {
        if constexpr (NI == 4) *(uint32_t*)row = word;
        else *(uint16_t*)row = (uint16_t)word;
      } else {  // byte by byte: the other slots of the row keep their contents
#pragma unroll
        for (int i = 0; i < NI; ++i)
          if (g * NI + i >= r_lo && g * NI + i < r_hi) row[i] = (uint8_t)(word >> (8 * i));
      }
    }
  }
}

// One run (the call's consecutive tokens that fall into one block: any start o_min, any length),
// K and V.  `done` comes back false, and nothing is written, if a block scale grows over older
// codes: they have to be re-expressed, which the general routine does.
template <int D>
__device__ inline void fp8_run_fast(const uint16_t* __restrict__ k_src,
                                    const uint16_t* __restrict__ v_src, size_t tstride,
                                    uint8_t* __restrict__ k_tile, uint8_t* __restrict__ v_tile,
                                    float* __restrict__ k_sp, float* __restrict__ v_sp, int o_min,
                                    int run, int bs, int lane, bool tensor_scale, bool& done) {
  constexpr int CL = D / 8, G = 64 / CL, NI = 16 / G;
  const int base0 = o_min & ~15;                       // block offset of the first sub-block touched
  const int nsb = ((o_min + run + 15) >> 4) - (o_min >> 4);
  // sub-block j of the run: its valid rows and where its first valid row's token lies
  auto rows_of = [&](int j, int& r_lo, int& r_hi, ptrdiff_t& first_token) {
    const int base = base0 + 16 * j;
    r_lo = max(o_min - base, 0);
    r_hi = min(o_min + run - base, 16);
    first_token = (ptrdiff_t)(base + r_lo - o_min);
  };
  // the first sub-block's rows stay in registers from the absmax pass to the encoding pass (a
  // block of 16 tokens is read once); further sub-blocks of the run are read again
  uint4 k_first[NI], v_first[NI];
  {
    int r_lo, r_hi;
    ptrdiff_t ft;
    rows_of(0, r_lo, r_hi, ft);
    load_subblock<D>(k_src + ft * (ptrdiff_t)tstride, tstride, 0, lane, r_lo, r_hi, k_first);
    load_subblock<D>(v_src + ft * (ptrdiff_t)tstride, tstride, 1, lane, r_lo, r_hi, v_first);
  }
  uint32_t amax[2] = {0, 0};
  if (!tensor_scale) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      amax[0] = max(amax[0], absmax8(k_first[i]));
      amax[1] = max(amax[1], absmax8(v_first[i]));
    }
    for (int j = 1; j < nsb; ++j) {
      int r_lo, r_hi;
      ptrdiff_t ft;
      rows_of(j, r_lo, r_hi, ft);
      uint4 a[NI], b[NI];
      load_subblock<D>(k_src + ft * (ptrdiff_t)tstride, tstride, 0, lane, r_lo, r_hi, a);
      load_subblock<D>(v_src + ft * (ptrdiff_t)tstride, tstride, 1, lane, r_lo, r_hi, b);
#pragma unroll
      for (int i = 0; i < NI; ++i) {
        amax[0] = max(amax[0], absmax8(a[i]));
        amax[1] = max(amax[1], absmax8(b[i]));
      }
    }
    amax[0] = wave_max_u32(amax[0]);
    amax[1] = wave_max_u32(amax[1]);
  }
  float s_new[2];
  done = true;
#pragma unroll
  for (int kv = 0; kv < 2; ++kv) {
    const float* sp = kv ? v_sp : k_sp;
    const float s_prev = (tensor_scale || o_min > 0) ? *sp : 0.0f;
    const float s_cand = (amax[kv] == 0) ? 0.0f : __fdiv_rn(bf16_bits_to_float(amax[kv]), 448.0f);
    s_new[kv] = s_prev > s_cand ? s_prev : s_cand;
    if (o_min > 0 && s_new[kv] > s_prev && s_prev > 0.0f) done = false;
  }
  if (!done) return;
  auto encode = [&](const uint4 (&raw)[NI], int kv, int j) {
    int r_lo, r_hi;
    ptrdiff_t ft;
    rows_of(j, r_lo, r_hi, ft);
    fp8_encode_subblock<D>(raw, kv, kv ? v_tile : k_tile, base0 + 16 * j, r_lo, r_hi, s_new[kv], bs,
                           lane);
  };
  encode(k_first, 0, 0);
  encode(v_first, 1, 0);
  for (int j = 1; j < nsb; ++j) {
    int r_lo, r_hi;
    ptrdiff_t ft;
    rows_of(j, r_lo, r_hi, ft);
    uint4 a[NI], b[NI];
    load_subblock<D>(k_src + ft * (ptrdiff_t)tstride, tstride, 0, lane, r_lo, r_hi, a);
    load_subblock<D>(v_src + ft * (ptrdiff_t)tstride, tstride, 1, lane, r_lo, r_hi, b);
    encode(a, 0, j);
    encode(b, 1, j);
  }
  if (lane == 0 && !tensor_scale) {
    *k_sp = s_new[0];
    *v_sp = s_new[1];
  }
}

// unit = (window of 16 consecutive tokens of the call, kv head): K and V, as for int8
template <int D>
__global__ __launch_bounds__(kWaves * 64) void write_fp8_bulk_kernel(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int64_t* __restrict__ slot_mapping, int32_t num_tokens, uint8_t* __restrict__ cache,
    float* __restrict__ scales, int32_t H, int32_t bs, int32_t tensor_scale) {
  const int lane = threadIdx.x & 63;
  const int64_t unit = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
  const int windows = (num_tokens + 15) >> 4;
  if (unit >= (int64_t)windows * H) return;
  const int h = (int)(unit % H);
  const int w0 = (int)(unit / H) * 16;
  // a run ends with its block, whose tokens share a scale; under static scales nothing ties a
  // block's sub-blocks together, so runs end with the sub-block and spread over more wavefronts
  const int span = tensor_scale ? 16 : bs;
  bool first = false;
  {
    const int t = w0 + lane;
    if (lane < 16 && t < num_tokens) {
      const int64_t slot = slot_mapping[t];
      if (slot >= 0)
        first = !(t > 0 && (slot & (span - 1)) > 0 && slot_mapping[t - 1] == slot - 1);
    }
  }
  uint32_t starts = (uint32_t)__ballot(first);
  const size_t tstride = (size_t)H * D;
  while (starts) {
    const int t0 = w0 + __builtin_ctz(starts);
    starts &= starts - 1;
    const int64_t slot0 = slot_mapping[t0];
    const int o_min = (int)(slot0 & (bs - 1));
    const int room = span - (int)(slot0 & (span - 1));  // slots left in the block / sub-block
    int run = 0;
    for (int base = 0; base < room; base += 64) {  // block sizes reach 256
      const int j = base + lane;
      const bool cont = j < room && t0 + j < num_tokens && slot_mapping[t0 + j] == slot0 + j;
      const unsigned long long m = __ballot(cont);
      const int n = m == ~0ull ? 64 : __builtin_ctzll(~m);
      run += n;
      if (n < 64) break;
    }
    const int64_t blk = slot0 >> __builtin_ctz(bs);
    const size_t row0 = ((size_t)t0 * H + h) * D;
    bool done = false;
    fp8_run_fast<D>(k + row0, v + row0, tstride, cache + tile_offset(blk, 0, h, H, bs, D),
                    cache + tile_offset(blk, 1, h, H, bs, D),
                    tensor_scale ? scales + 0 : scales + ((size_t)blk * 2 + 0) * H + h,
                    tensor_scale ? scales + 1 : scales + ((size_t)blk * 2 + 1) * H + h, o_min, run,
                    bs, lane, tensor_scale != 0, done);
    if (!done) {
      fp8_run<D>(k, v, cache, scales, H, bs, 0, h, t0, slot0, run, lane, tensor_scale != 0);
      fp8_run<D>(k, v, cache, scales, H, bs, 1, h, t0, slot0, run, lane, tensor_scale != 0);
    }
  }
}

// Blocks of more than 16 tokens under one scale per block: the block's absmax ties its
// sub-blocks together, and one wavefront doing them one after the other (as above) leaves the
// wavefronts of the block's other windows with nothing to do.  Here a workgroup of bs / 16
// wavefronts owns bs consecutive tokens of the call and one kv head, and handles the runs that
// start among them: wavefront j loads sub-block j of the run (K and V, kept in registers),
// the sub-blocks' absmax values meet in LDS, and every wavefront encodes its own sub-block
// under the block's scale.  A run whose scale would grow over older codes of the block goes to
// the general routine (wavefront 0), as above.  Every wavefront takes every barrier: the list
// of runs comes from LDS and the loops over it are uniform.
template <int D>
__global__ __launch_bounds__(1024) void write_fp8_block_kernel(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int64_t* __restrict__ slot_mapping, int32_t num_tokens, uint8_t* __restrict__ cache,
    float* __restrict__ scales, int32_t H, int32_t bs) {
  constexpr int CL = D / 8, G = 64 / CL, NI = 16 / G;
  __shared__ uint32_t sh_starts[16];
  __shared__ uint32_t sh_amax[2][16];
  __shared__ float sh_prev[2];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int nw = bs >> 4;  // wavefronts of the workgroup = sub-blocks of a block
  const int h = (int)(blockIdx.x % H);
  const int g0 = (int)(blockIdx.x / H) * bs;  // the workgroup's first token
  {
    bool first = false;
    const int t = g0 + 16 * wv + lane;
    if (lane < 16 && t < num_tokens) {
      const int64_t slot = slot_mapping[t];
      if (slot >= 0)
        first = !(t > 0 && (slot & (bs - 1)) > 0 && slot_mapping[t - 1] == slot - 1);
    }
    const uint32_t starts = (uint32_t)__ballot(first);
    if (lane == 0) sh_starts[wv] = starts;
  }
  __syncthreads();
  const size_t tstride = (size_t)H * D;
  for (int ww = 0; ww < nw; ++ww) {
    uint32_t starts = sh_starts[ww];
    while (starts) {
      const int t0 = g0 + 16 * ww + __builtin_ctz(starts);
      starts &= starts - 1;
      const int64_t slot0 = slot_mapping[t0];
      const int o_min = (int)(slot0 & (bs - 1));
      const int room = bs - o_min;  // slots left in the block
      int run = 0;
      for (int base = 0; base < room; base += 64) {  // block sizes reach 256
        const int j = base + lane;
        const bool cont = j < room && t0 + j < num_tokens && slot_mapping[t0 + j] == slot0 + j;
        const unsigned long long m = __ballot(cont);
        const int n = m == ~0ull ? 64 : __builtin_ctzll(~m);
        run += n;
        if (n < 64) break;
      }
      const int64_t blk = slot0 >> __builtin_ctz(bs);
      float* k_sp = scales + ((size_t)blk * 2 + 0) * H + h;
      float* v_sp = scales + ((size_t)blk * 2 + 1) * H + h;
      // this wavefront's sub-block of the run: its valid rows, where its first valid row's
      // token lies
      const int base0 = o_min & ~15;
      const int nsb = ((o_min + run + 15) >> 4) - (o_min >> 4);
      const bool mine = wv < nsb;
      const int base = base0 + 16 * wv;
      const int r_lo = max(o_min - base, 0), r_hi = min(o_min + run - base, 16);
      uint4 k_rows[NI], v_rows[NI];
      uint32_t amax_k = 0, amax_v = 0;
      if (mine) {
        const size_t row = ((size_t)(t0 + (base + r_lo - o_min)) * H + h) * D;
        load_subblock<D>(k + row, tstride, 0, lane, r_lo, r_hi, k_rows);
        load_subblock<D>(v + row, tstride, 1, lane, r_lo, r_hi, v_rows);
#pragma unroll
        for (int i = 0; i < NI; ++i) {
          amax_k = max(amax_k, absmax8(k_rows[i]));
          amax_v = max(amax_v, absmax8(v_rows[i]));
        }
        amax_k = wave_max_u32(amax_k);
        amax_v = wave_max_u32(amax_v);
      }
      if (lane == 0) {
        sh_amax[0][wv] = amax_k;
        sh_amax[1][wv] = amax_v;
        if (wv == 0) {  // the block's scales before this run (a run from offset 0 starts afresh)
          sh_prev[0] = o_min > 0 ? *k_sp : 0.0f;
          sh_prev[1] = o_min > 0 ? *v_sp : 0.0f;
        }
      }
      __syncthreads();
      float s_new[2];
      bool done = true;
#pragma unroll
      for (int kv = 0; kv < 2; ++kv) {
        uint32_t amax = 0;
        for (int j = 0; j < nw; ++j) amax = max(amax, sh_amax[kv][j]);
        const float s_prev = sh_prev[kv];
        const float s_cand = (amax == 0) ? 0.0f : __fdiv_rn(bf16_bits_to_float(amax), 448.0f);
        s_new[kv] = s_prev > s_cand ? s_prev : s_cand;
        if (o_min > 0 && s_new[kv] > s_prev && s_prev > 0.0f) done = false;
      }
      if (done) {
        if (mine) {
          fp8_encode_subblock<D>(k_rows, 0, cache + tile_offset(blk, 0, h, H, bs, D), base, r_lo, r_hi,
                                 s_new[0], bs, lane);
          fp8_encode_subblock<D>(v_rows, 1, cache + tile_offset(blk, 1, h, H, bs, D), base, r_lo, r_hi,
                                 s_new[1], bs, lane);
        }
        if (wv == 0 && lane == 0) {
          *k_sp = s_new[0];
          *v_sp = s_new[1];
        }
      } else if (wv == 0) {
        fp8_run<D>(k, v, cache, scales, H, bs, 0, h, t0, slot0, run, lane, false);
        fp8_run<D>(k, v, cache, scales, H, bs, 1, h, t0, slot0, run, lane, false);
      }
      __syncthreads();  // (the LDS words are written again for the next run)
    }
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
// GROUPED: one scale per 32 adjacent channels (the 16 lanes of a row own them) instead of one
// per token and head; the scales of a token are then 4 adjacent floats.
template <bool GROUPED>
__device__ inline void int4_run(const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                                uint8_t* __restrict__ cache, float* __restrict__ scales, int H,
                                int bs, int kv, int h, int t0, int64_t slot0, int run, int lane) {
  constexpr int D = 128, NG = GROUPED ? 4 : 1;
  const int64_t blk = slot0 >> __builtin_ctz(bs);
  const int off0 = (int)(slot0 - blk * bs);
  const int so = off0 & 15;
  uint8_t* tile = cache + (size_t)tile_offset(blk, kv, h, H, bs, D / 2);
  float* srow = scales + ((((size_t)blk * 2 + kv) * H + h) * bs + off0) * NG;
  const uint16_t* src = (kv ? v : k) + ((size_t)t0 * H + h) * D + lane * 2;
  const size_t tstride = (size_t)H * D;
  unsigned long long img[2] = {0, 0}, mask = 0;  // V rows of the lane's two channels
  for (int i = 0; i < run; ++i) {
    const uint32_t w = *(const uint32_t*)(src + i * tstride);
    const uint32_t b0 = w & 0xFFFFu, b1 = w >> 16;
    uint32_t amax = (b0 & 0x7FFFu) > (b1 & 0x7FFFu) ? (b0 & 0x7FFFu) : (b1 & 0x7FFFu);
    amax = GROUPED ? row_max_u32<16>(amax) : wave_max_u32(amax);
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
    if (GROUPED ? (lane & 15) == 0 : lane == 0) srow[i * NG + (GROUPED ? lane >> 4 : 0)] = s;
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

template <bool GROUPED>
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
  int4_run<GROUPED>(k, v, cache, scales, H, bs, kv, h, t0, slot0, run, lane);
}

// A whole sub-block with 16-byte loads, as for int8: a lane owns 8 channels (8 c .. 8 c + 7,
// c = lane % 16) of 4 tokens.  K (tokens 4 i + g): the lane's eight codes of a token are one
// whole word.  V (tokens 4 g + i): the lane's four tokens of a channel are the nibbles
// 2a, 2a+1 (one byte) and 2a+4, 2a+5 (another byte) of the channel's word g / 2, a = g % 2.
template <bool GROUPED>
__device__ inline void int4_subblock(const uint16_t* __restrict__ src, size_t tstride,
                                     uint8_t* __restrict__ tile, float* __restrict__ srow,
                                     int kv, int off0, int lane) {
  constexpr int NG = GROUPED ? 4 : 1;  // scales per token; a group of 32 channels = 4 lanes
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
    amax = GROUPED ? row_max_u32<4>(amax) : row_max_u32<16>(amax);
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
    if (GROUPED ? (c & 3) == 0 : c == 0) srow[tok[i] * NG + (GROUPED ? c >> 2 : 0)] = s;
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

template <bool GROUPED>
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
      int4_subblock<GROUPED>((kv ? v : k) + ((size_t)t0 * H + h) * D, tstride,
                             cache + (size_t)tile_offset(blk, kv, h, H, bs, D / 2),
                             scales + ((((size_t)blk * 2 + kv) * H + h) * bs + off0) * (GROUPED ? 4 : 1),
                             kv, off0, lane);
    } else {
      int4_run<GROUPED>(k, v, cache, scales, H, bs, kv, h, t0, slot0, run, lane);
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
  if (is_int4(desc.mode)) {
    const bool grouped = desc.mode == KVQ_INT4_GROUP32;
    if (bulk && grouped)
      hipLaunchKernelGGL(write_int4_bulk_kernel<true>, dim3(grid), block, 0, stream, kk, vv, slot_mapping,
                         num_tokens, c, scales, desc.num_kv_heads, desc.block_size);
    else if (bulk)
      hipLaunchKernelGGL(write_int4_bulk_kernel<false>, dim3(grid), block, 0, stream, kk, vv, slot_mapping,
                         num_tokens, c, scales, desc.num_kv_heads, desc.block_size);
    else if (grouped)
      hipLaunchKernelGGL(write_int4_kernel<true>, dim3(grid), block, 0, stream, kk, vv, slot_mapping,
                         num_tokens, c, scales, desc.num_kv_heads, desc.block_size);
    else
      hipLaunchKernelGGL(write_int4_kernel<false>, dim3(grid), block, 0, stream, kk, vv, slot_mapping,
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
    // (a wavefront of this kernel handles K and V: half the units)
    const unsigned g = (unsigned)((units / 2 + kWaves - 1) / kWaves);
    if (desc.head_dim == 128)
      hipLaunchKernelGGL((write_int8_bulk_kernel<128>), dim3(g), block, 0, stream, kk, vv, slot_mapping,
                         num_tokens, c, scales, desc.num_kv_heads, desc.block_size);
    else
      hipLaunchKernelGGL((write_int8_bulk_kernel<64>), dim3(g), block, 0, stream, kk, vv, slot_mapping,
                         num_tokens, c, scales, desc.num_kv_heads, desc.block_size);
  } else if (bulk && desc.mode == KVQ_FP8E4M3_BLOCK_HEAD && desc.block_size > 16) {
    // a workgroup per (block_size consecutive tokens, head), a wavefront per sub-block
    const int64_t groups = ((int64_t)num_tokens + desc.block_size - 1) / desc.block_size;
    const dim3 grid((unsigned)(groups * desc.num_kv_heads)), wg((unsigned)(desc.block_size / 16 * 64));
    if (desc.head_dim == 128)
      hipLaunchKernelGGL((write_fp8_block_kernel<128>), grid, wg, 0, stream, kk, vv, slot_mapping,
                         num_tokens, c, scales, desc.num_kv_heads, desc.block_size);
    else
      hipLaunchKernelGGL((write_fp8_block_kernel<64>), grid, wg, 0, stream, kk, vv, slot_mapping,
                         num_tokens, c, scales, desc.num_kv_heads, desc.block_size);
  } else if (bulk) {
    const unsigned g = (unsigned)((units / 2 + kWaves - 1) / kWaves);  // K and V per wavefront
    const int32_t ts = desc.mode == KVQ_FP8E4M3_TENSOR;
    if (desc.head_dim == 128)
      hipLaunchKernelGGL((write_fp8_bulk_kernel<128>), dim3(g), block, 0, stream, kk, vv, slot_mapping,
                         num_tokens, c, scales, desc.num_kv_heads, desc.block_size, ts);
    else
      hipLaunchKernelGGL((write_fp8_bulk_kernel<64>), dim3(g), block, 0, stream, kk, vv, slot_mapping,
                         num_tokens, c, scales, desc.num_kv_heads, desc.block_size, ts);
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
