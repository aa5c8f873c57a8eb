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

// ---- int8, one scale per (token, kv head) -------------------------------------------------
template <int D>
__global__ __launch_bounds__(kWaves * 64) void write_int8_kernel(
    const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    const int64_t* __restrict__ slot_mapping, int32_t num_tokens, uint8_t* __restrict__ cache,
    float* __restrict__ scales, int32_t H, int32_t bs) {
  constexpr int E = D / 64;  // elements per lane
  const int lane = threadIdx.x & 63;
  const int64_t unit = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
  if (unit >= (int64_t)num_tokens * H * 2) return;
  const int kv = (int)(unit & 1);
  const int h = (int)((unit >> 1) % H);
  const int t = (int)((unit >> 1) / H);
  const int64_t slot = slot_mapping[t];
  if (slot < 0) return;
  const int64_t blk = slot / bs;
  const int off = (int)(slot - blk * bs);

  const uint16_t* row = (kv ? v : k) + ((size_t)t * H + h) * D + lane * E;
  uint32_t bits[E];
  uint32_t amax = 0;
#pragma unroll
  for (int e = 0; e < E; ++e) {
    bits[e] = row[e];
    const uint32_t a = bits[e] & 0x7FFF;
    amax = a > amax ? a : amax;
  }
  amax = wave_max_u32(amax);  // |bf16| orders like its bit pattern
  const float m = bf16_bits_to_float(amax);
  const float s = (amax == 0) ? 0.0f : (float)((double)m / 127.0);

  uint8_t* tile = cache + tile_offset(blk, kv, h, H, bs, D);
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const int d = lane * E + e;
    const uint8_t c = (amax == 0) ? (uint8_t)0 : int8_code(bf16_bits_to_float(bits[e]), s);
    tile[kv ? v_elem(off, d, bs, D) : k_elem(off, d, bs, D)] = stored_byte(c, KVQ_INT8_TOKEN_HEAD);
  }
  if (lane == 0) scales[(((size_t)blk * 2 + kv) * H + h) * bs + off] = s;
}

// ---- fp8-e4m3, one scale per (block, kv head) ---------------------------------------------
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
  // Only the first token of a run works: the previous token continues into this slot?
  if (t0 > 0 && o_min > 0 && slot_mapping[t0 - 1] == slot0 - 1) return;
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

  uint8_t* tile = cache + tile_offset(blk, kv, h, H, bs, D);
  if (o_min > 0 && s_new > s_prev && s_prev > 0.0f) {
    // the block's scale grew: re-express the codes stored below the run in the new scale
    for (int off = 0; off < o_min; ++off) {
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const int d = lane * E + e;
        uint8_t* pc = tile + (kv ? v_elem(off, d, bs, D) : k_elem(off, d, bs, D));
        const uint32_t c = *pc;
        if ((c & 0x7F) == 0x7F) continue;  // NaN codes stay
        *pc = fp8_code(fp8_value(c) * (double)s_prev / (double)s_new);
      }
    }
  }
  for (int i = 0; i < run; ++i) {
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const int d = lane * E + e;
      uint8_t c = 0;
      if (s_new > 0.0f)
        c = fp8_code((double)bf16_bits_to_float(src[i * tstride + e]) / (double)s_new);
      tile[kv ? v_elem(o_min + i, d, bs, D) : k_elem(o_min + i, d, bs, D)] = c;
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
