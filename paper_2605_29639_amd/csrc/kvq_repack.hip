// Conversions between the library's physical cache (K in 4-token quads, V channel-major per
// 16-token sub-block, int8 codes in offset-binary form) and the canonical
// [block][K|V][head][token][channel] array of plain codes.  Not on the hot
// path: used to hand a cache to, or take one from, code that expects the canonical order.
#include "kvq_internal.h"

namespace kvq {
namespace {

typedef uint32_t uintx4v __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void repack_kernel(const uint8_t* __restrict__ src,
                                                     uint8_t* __restrict__ dst, size_t total,
                                                     int H, int bs, int D, int mode,
                                                     bool to_canonical) {
  const size_t tile_bytes = (size_t)bs * D;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (size_t)gridDim.x * blockDim.x) {
    // i indexes the canonical array
    const size_t tile = i / tile_bytes;
    const int within = (int)(i - tile * tile_bytes);
    const int off = within / D, d = within - off * D;
    const int kv = (int)((tile / H) & 1);
    const size_t phys = tile * tile_bytes + (kv ? v_elem(off, d, bs, D) : k_elem(off, d, bs, D));
    // stored_byte is its own inverse
    if (to_canonical) dst[i] = stored_byte(src[phys], mode);
    else dst[phys] = stored_byte(src[i], mode);
  }
}

// int4 (head_dim 128): canonical byte j of a token = channels 2j (low nibble) and 2j+1 (high),
// 4-bit two's complement; physical nibble = code + 8 in the word / nibble given by
// int4_k_word / int4_v_word / int4_nibble.  One thread per canonical byte when converting to
// the canonical form (it gathers two nibbles), one per physical 32-bit word the other way (it
// gathers eight), so every output location has exactly one writer.
__global__ __launch_bounds__(256) void repack_int4_kernel(const uint8_t* __restrict__ src,
                                                          uint8_t* __restrict__ dst, size_t total,
                                                          int H, int bs, bool to_canonical) {
  constexpr int D = 128;
  const size_t tile_bytes = (size_t)bs * (D / 2);
  if (to_canonical) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (size_t)gridDim.x * blockDim.x) {
      const size_t tile = i / tile_bytes;
      const int within = (int)(i - tile * tile_bytes);
      const int off = within / (D / 2), j = within - off * (D / 2);
      const int kv = (int)((tile / H) & 1);
      uint32_t byte = 0;
      for (int half = 0; half < 2; ++half) {
        const int d = 2 * j + half;
        const int word = kv ? int4_v_word(off, d) : int4_k_word(off, d);
        const int nib = int4_nibble(kv ? (off & 7) : (d & 7));
        const uint32_t w = *(const uint32_t*)(src + tile * tile_bytes + word);
        const uint32_t code = (((w >> (4 * nib)) & 15u) - 8u) & 15u;
        byte |= code << (4 * half);
      }
      dst[i] = (uint8_t)byte;
    }
  } else {
    const size_t words = total / 4;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < words;
         i += (size_t)gridDim.x * blockDim.x) {
      const size_t tile = (i * 4) / tile_bytes;
      const int word = (int)(i * 4 - tile * tile_bytes);
      const int kv = (int)((tile / H) & 1);
      uint32_t w = 0;
      for (int e = 0; e < 8; ++e) {
        int off, d;
        if (kv == 0) {  // invert int4_k_word: the word's token and its 8 channels
          off = (word >> 8) * 4 + ((word >> 4) & 3);
          d = ((word >> 2) & 3) * 32 + ((word >> 6) & 3) * 8 + e;
        } else {        // invert int4_v_word: the word's channel and its 8 tokens
          off = (word >> 10) * 16 + ((word >> 2) & 1) * 8 + e;
          d = ((word >> 8) & 3) * 32 + ((word >> 3) & 1) * 16 + ((word >> 4) & 15);
        }
        const uint32_t byte = src[tile * tile_bytes + (size_t)off * (D / 2) + d / 2];
        const uint32_t code = (d & 1) ? (byte >> 4) : (byte & 15u);
        w |= ((code + 8u) & 15u) << (4 * int4_nibble(e));
      }
      *(uint32_t*)(dst + tile * tile_bytes + word) = w;
    }
  }
}

__global__ __launch_bounds__(256) void repack16_kernel(const uint16_t* __restrict__ src,
                                                       uint16_t* __restrict__ dst, size_t total,
                                                       int H, int bs, int D, bool to_canonical) {
  const size_t tile_elems = (size_t)bs * D;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (size_t)gridDim.x * blockDim.x) {
    const size_t tile = i / tile_elems;
    const int within = (int)(i - tile * tile_elems);
    const int off = within / D, d = within - off * D;
    const int kv = (int)((tile / H) & 1);
    const size_t phys = tile * tile_elems + (kv ? v_elem16(off, d, D) : k_elem16(off, d, D));
    if (to_canonical) dst[i] = src[phys];
    else dst[phys] = src[i];
  }
}

// Whole blocks between the pool and a packed staging area.  A workgroup moves one 4 KiB piece
// of one block's codes (16 bytes per lane); the workgroup of a block's first piece also moves
// the block's scales.  Non-temporal on both sides: every byte is touched once.
__global__ __launch_bounds__(256) void block_copy_kernel(
    uint8_t* __restrict__ pool_cache, float* __restrict__ pool_scales,
    uint8_t* __restrict__ packed_cache, float* __restrict__ packed_scales,
    const int32_t* __restrict__ block_ids, uint32_t block_bytes, uint32_t scale_floats,
    uint32_t pieces, bool to_packed) {
  const uint32_t i = blockIdx.x / pieces, piece = blockIdx.x - i * pieces;
  const size_t blk = (size_t)block_ids[i];
  const uint32_t at = piece * 4096u + threadIdx.x * 16u;
  if (at < block_bytes) {
    uintx4v* in_pool = (uintx4v*)(pool_cache + blk * block_bytes + at);
    uintx4v* in_packed = (uintx4v*)(packed_cache + (size_t)i * block_bytes + at);
    if (to_packed) __builtin_nontemporal_store(__builtin_nontemporal_load(in_pool), in_packed);
    else __builtin_nontemporal_store(__builtin_nontemporal_load(in_packed), in_pool);
  }
  if (piece == 0) {
    for (uint32_t k = threadIdx.x; k < scale_floats; k += 256) {
      float* in_pool = pool_scales + blk * scale_floats + k;
      float* in_packed = packed_scales + (size_t)i * scale_floats + k;
      if (to_packed) *in_packed = *in_pool;
      else *in_pool = *in_packed;
    }
  }
}

}  // namespace

hipError_t launch_block_copy(const void* pool_cache, const float* pool_scales,
                             const kvq_cache_desc_t& desc, const int32_t* block_ids, int32_t num,
                             void* packed_cache, float* packed_scales, bool to_packed,
                             hipStream_t stream) {
  const uint32_t block_bytes =
      2u * desc.num_kv_heads * desc.block_size * row_bytes(desc.mode, desc.head_dim);
  const uint32_t scale_floats = (uint32_t)block_scale_floats(desc.mode, desc.num_kv_heads,
                                                             desc.block_size, desc.head_dim);
  const uint32_t pieces = (block_bytes + 4095u) / 4096u;
  hipLaunchKernelGGL(block_copy_kernel, dim3((unsigned)num * pieces), dim3(256), 0, stream,
                     (uint8_t*)pool_cache, (float*)pool_scales, (uint8_t*)packed_cache,
                     packed_scales, block_ids, block_bytes, scale_floats, pieces, to_packed);
  return hipGetLastError();
}

hipError_t launch_repack(const void* src, void* dst, const kvq_cache_desc_t& desc,
                         bool to_canonical, hipStream_t stream) {
  const size_t total = (size_t)desc.num_blocks * 2 * desc.num_kv_heads * desc.block_size *
                       (is_int4(desc.mode) ? desc.head_dim / 2 : desc.head_dim);
  if (total == 0) return hipSuccess;
  size_t blocks = (total + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  if (is_int4(desc.mode)) {
    hipLaunchKernelGGL(repack_int4_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                       (const uint8_t*)src, (uint8_t*)dst, total, desc.num_kv_heads,
                       desc.block_size, to_canonical);
    return hipGetLastError();
  }
  if (desc.mode == KVQ_BF16_PLAIN) {
    hipLaunchKernelGGL(repack16_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                       (const uint16_t*)src, (uint16_t*)dst, total, desc.num_kv_heads,
                       desc.block_size, desc.head_dim, to_canonical);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(repack_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                     (const uint8_t*)src, (uint8_t*)dst, total, desc.num_kv_heads,
                     desc.block_size, desc.head_dim, desc.mode, to_canonical);
  return hipGetLastError();
}

}  // namespace kvq
