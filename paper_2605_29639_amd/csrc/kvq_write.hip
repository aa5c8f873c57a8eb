// kv_quant_write kernels (gfx950): bf16 K/V rows -> int8 or fp8-e4m3 codes + fp32 scales in
// the paged cache (Section 7.2.2, on-the-fly quantization with dynamic scaling).
//
// One 64-lane wavefront owns one unit of work, so every output byte and every scale has
// exactly one writer and no atomics are needed:
//   int8 per (token, head): unit = (token, kv head, K|V) row of head_dim values;
//   fp8 per (block, head):  unit = (run, kv head, K|V), a run being the consecutive tokens
//                           of the call that fall into one cache block.
// The decisions that fix an integer (the rounding of x/scale) are taken in fp64: for a bf16
// x and an fp32 scale the fp64 quotient is either exactly a rounding tie or at least 2^-25
// (relative 2^-29 for the fp8 midpoints) away from one, so rounding it equals rounding the
// exact quotient.  The scale itself is the fp64 quotient absmax/qmax rounded once to fp32.
#include "kvq_internal.h"

namespace kvq {
namespace {

constexpr int kWaves = 4;  // wavefronts per workgroup

__device__ inline float bf16_bits_to_float(uint32_t bits16) {
  return __uint_as_float(bits16 << 16);
}

__device__ inline uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) {
    uint32_t o = (uint32_t)__shfl_xor((int)v, s, 64);
    v = v > o ? v : o;
  }
  return v;
}

__device__ inline uint8_t int8_code(float x, float s) {
  double r = rint((double)x / (double)s);  // v_rndne_f64: ties to even
  r = r > 127.0 ? 127.0 : r;
  r = r < -127.0 ? -127.0 : r;
  return (uint8_t)(int8_t)(int)r;
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
// sub-block with consecutive slots; the wavefront of the run's first token does the work.
template <int D>
__global__ __launch_bounds__(kWaves * 64) void write_int8_kernel(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int64_t* __restrict__ slot_mapping, int32_t num_tokens, uint8_t* __restrict__ cache,
    float* __restrict__ scales, int32_t H, int32_t bs) {
  constexpr int E = D / 64;  // channels per lane
  const int lane = threadIdx.x & 63;
  const int64_t unit = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
  if (unit >= (int64_t)num_tokens * H * 2) return;
  const int kv = (int)(unit & 1);
  const int h = (int)((unit >> 1) % H);
  const int t0 = (int)((unit >> 1) / H);
  const int64_t slot0 = slot_mapping[t0];
  if (slot0 < 0) return;
  const int64_t blk = slot0 / bs;
  const int off0 = (int)(slot0 - blk * bs);
  const int so = off0 & 15;  // position inside the sub-block
  if (t0 > 0 && so > 0 && slot_mapping[t0 - 1] == slot0 - 1) return;  // not a run's first token
  int run = 1;
  while (run < 16 - so && t0 + run < num_tokens && slot_mapping[t0 + run] == slot0 + run) ++run;

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

// ---- fp8-e4m3, one scale per (block, kv head) ---------------------------------------------
// unit = (run, kv head, K|V): the consecutive tokens of the call that fall into one block.
template <int D>
__global__ __launch_bounds__(kWaves * 64) void write_fp8_kernel(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int64_t* __restrict__ slot_mapping, int32_t num_tokens, uint8_t* __restrict__ cache,
    float* __restrict__ scales, int32_t H, int32_t bs) {
  constexpr int E = D / 64;
  const int lane = threadIdx.x & 63;
  const int64_t unit = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
  if (unit >= (int64_t)num_tokens * H * 2) return;
  const int kv = (int)(unit & 1);
  const int h = (int)((unit >> 1) % H);
  const int t0 = (int)((unit >> 1) / H);
  const int64_t slot0 = slot_mapping[t0];
  if (slot0 < 0) return;
  const int64_t blk = slot0 / bs;
  const int o_min = (int)(slot0 - blk * bs);
  if (t0 > 0 && o_min > 0 && slot_mapping[t0 - 1] == slot0 - 1) return;  // not a run's first token
  int run = 1;
  while (run < bs - o_min && t0 + run < num_tokens && slot_mapping[t0 + run] == slot0 + run) ++run;

  const uint16_t* src = (kv ? v : k) + ((size_t)t0 * H + h) * D + lane * E;
  const size_t tstride = (size_t)H * D;
  uint32_t amax = 0;
  for (int i = 0; i < run; ++i) {
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const uint32_t a = src[i * tstride + e] & 0x7FFF;
      amax = a > amax ? a : amax;
    }
  }
  amax = wave_max_u32(amax);
  float* sp = scales + ((size_t)blk * 2 + kv) * H + h;
  const float s_prev = (o_min > 0) ? *sp : 0.0f;
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
  if (lane == 0) *sp = s_new;
}

}  // namespace

hipError_t launch_write(const void* k, const void* v, const int64_t* slot_mapping,
                        int32_t num_tokens, void* cache, float* scales,
                        const kvq_cache_desc_t& desc, hipStream_t stream) {
  const int64_t units = (int64_t)num_tokens * desc.num_kv_heads * 2;
  const unsigned grid = (unsigned)((units + kWaves - 1) / kWaves);
  const dim3 block(kWaves * 64);
  const uint16_t* kk = (const uint16_t*)k;
  const uint16_t* vv = (const uint16_t*)v;
  uint8_t* c = (uint8_t*)cache;
#define KVQ_LAUNCH_WRITE(KERNEL, DD)                                                          \
  hipLaunchKernelGGL((KERNEL<DD>), dim3(grid), block, 0, stream, kk, vv, slot_mapping,        \
                     num_tokens, c, scales, desc.num_kv_heads, desc.block_size)
  if (desc.mode == KVQ_INT8_TOKEN_HEAD) {
    if (desc.head_dim == 128) KVQ_LAUNCH_WRITE(write_int8_kernel, 128);
    else KVQ_LAUNCH_WRITE(write_int8_kernel, 64);
  } else {
    if (desc.head_dim == 128) KVQ_LAUNCH_WRITE(write_fp8_kernel, 128);
    else KVQ_LAUNCH_WRITE(write_fp8_kernel, 64);
  }
#undef KVQ_LAUNCH_WRITE
  return hipGetLastError();
}

}  // namespace kvq
