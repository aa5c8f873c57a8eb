// Internal declarations shared by the library's translation units (host side).
// The device kernels live in kvq_write.hip, kvq_attn.hip and kvq_repack.hip; kvq_api.hip
// holds the extern "C" entry points, which validate on the host and then call these.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/kvq.h"

namespace kvq {

// Physical position of the (blk, kv, h) tile inside the cache buffer, in bytes.
__host__ __device__ inline size_t tile_offset(int64_t blk, int kv, int h, int num_kv_heads,
                                              int block_size, int head_dim) {
  return (((size_t)blk * 2 + (size_t)kv) * (size_t)num_kv_heads + (size_t)h) *
         (size_t)block_size * (size_t)head_dim;
}
// Position of logical element (off, d) inside a (block, K|V, head) tile.  Both orders are
// chosen so that the 16-byte piece one lane feeds to a matrix instruction is contiguous and
// the four lanes of a quad read 64 contiguous bytes:
//   K: quads of 4 tokens; inside a quad, 16-channel slices, then the 4 tokens, then 16 channels
//   V: sub-blocks of 16 tokens; inside one, channel-major rows of 16 tokens
__host__ __device__ inline int k_elem(int off, int d, int /*block_size*/, int head_dim) {
  return (off >> 2) * (4 * head_dim) + (d >> 4) * 64 + (off & 3) * 16 + (d & 15);
}
__host__ __device__ inline int v_elem(int off, int d, int /*block_size*/, int head_dim) {
  return (off >> 4) * (16 * head_dim) + d * 16 + (off & 15);
}

// The same two orders for the 2-byte elements of an unquantized cache, in elements: a lane's
// 16-byte piece is 8 elements, so K slices are 8 channels wide and a V row of 16 tokens is
// kept as two half-rows of 8 (all channels' first halves, then all second halves).
__host__ __device__ inline int k_elem16(int off, int d, int head_dim) {
  return (off >> 2) * (4 * head_dim) + (d >> 3) * 32 + (off & 3) * 8 + (d & 7);
}
__host__ __device__ inline int v_elem16(int off, int d, int head_dim) {
  return (off >> 4) * (16 * head_dim) + ((off >> 3) & 1) * (8 * head_dim) + d * 8 + (off & 7);
}
__host__ __device__ inline int elem_bytes(int mode) { return mode == KVQ_BF16_PLAIN ? 2 : 1; }
__host__ __device__ inline bool is_int4(int mode) {
  return mode == KVQ_INT4_TOKEN_HEAD || mode == KVQ_INT4_GROUP32;
}
// bytes one token's head_dim values take in the cache
__host__ __device__ inline int row_bytes(int mode, int head_dim) {
  return mode == KVQ_BF16_PLAIN ? 2 * head_dim : is_int4(mode) ? head_dim / 2 : head_dim;
}
// fp32 scales that belong to one block of the pool (0: the format's scales are not per block)
__host__ __device__ inline size_t block_scale_floats(int mode, int num_kv_heads, int block_size,
                                                     int head_dim) {
  const size_t token_heads = (size_t)2 * num_kv_heads * block_size;
  return mode == KVQ_INT8_TOKEN_HEAD || mode == KVQ_INT4_TOKEN_HEAD ? token_heads
         : mode == KVQ_INT4_GROUP32      ? token_heads * (head_dim / 32)
         : mode == KVQ_FP8E4M3_BLOCK_HEAD ? (size_t)2 * num_kv_heads
                                          : 0;
}

// int4 (head_dim 128): byte offset, inside a tile, of the 32-bit word that holds logical element
// (off, d), and the nibble of that word it sits in.  A word holds the 8 codes one lane feeds to
// one matrix instruction (K: 8 channels of a token; V: 8 tokens of a channel), element e of the
// 8 in nibble e/2 (even e) or e/2 + 4 (odd e).
__host__ __device__ inline int int4_k_word(int off, int d) {
  return (off >> 2) * 256 + ((d & 31) >> 3) * 64 + (off & 3) * 16 + (d >> 5) * 4;
}
__host__ __device__ inline int int4_v_word(int off, int d) {
  return (off >> 4) * 1024 + (d >> 5) * 256 + (d & 15) * 16 + ((d >> 4) & 1) * 8 +
         ((off >> 3) & 1) * 4;
}
__host__ __device__ inline int int4_nibble(int e) { return (e >> 1) + ((e & 1) << 2); }

// int8 codes are kept in the cache in offset-binary form (stored byte = code XOR 0x80, i.e.
// code + 128), which is the form the byte -> f16 conversion in the attention kernel consumes
// directly; e4m3 codes are stored as they are.
__host__ __device__ inline uint8_t stored_byte(uint8_t code, int mode) {
  return mode == KVQ_INT8_TOKEN_HEAD ? (uint8_t)(code ^ 0x80) : code;
}

constexpr int kMaxPrefixChunks = 8;  // pieces a shared prefix is cut into at most

struct AttnPlan {
  int32_t rows;            // (num_q_heads / num_kv_heads) * q_len query rows per kv head
  int32_t row_tiles;       // 16-row tiles handled by one wavefront (1 or 2)
  int32_t num_row_groups;  // ceil(rows / (16 * row_tiles))
  int32_t pairs_per_seq;   // num_kv_heads * num_row_groups
  int32_t range_groups;    // 64-token groups per wavefront range; 0 = even split on the device
  int32_t num_waves;       // wavefronts launched (= grid size)
  size_t acc_floats;       // workspace: accumulators
  size_t ml_floats;        // workspace: (max, sum) pairs
  size_t prefix_ints;      // workspace: groups before each sequence and the prefix length (batch + 2, padded to 4)
  int32_t shared_groups;   // shared prefix in 64-token groups, 0 where the prefix kernel is not used
  int32_t prefix_chunks;   // pieces the prefix kernel cuts it into (>= 1)
};

struct AttnArgs {
  const uint16_t* q;
  const uint8_t* cache;
  const float* scales;
  const int32_t* block_tables;
  const int32_t* seq_lens;
  float* out;
  float* ws_acc;
  float* ws_ml;
  int32_t* ws_prefix;  // [batch + 1] 64-token groups of the sequences before b, then the shared
                       // prefix length in groups that the streaming kernel split off (written
                       // by its first wavefront, read by the reduce)
  int32_t max_blocks_per_seq, batch, q_len, num_q_heads, num_kv_heads, group, rows;
  int32_t block_size, bs_shift, head_dim, mode;
  int32_t row_tiles, num_row_groups, pairs_per_seq, range_groups, num_waves;
  float scale_log2;  // sm_scale * log2(e)
  int32_t shared_groups;  // leading 64-token groups that all sequences' tables map to the same
                          // blocks (0: none, or a call the prefix kernel does not serve)
  int32_t prefix_chunks;  // pieces the prefix kernel cuts those groups into: one partial each
  unsigned long long* wave_clock;  // measurement build: 8 clock readings per wavefront; else null
};

hipError_t launch_write(const void* k, const void* v, const int64_t* slot_mapping,
                        int32_t num_tokens, void* cache, float* scales,
                        const kvq_cache_desc_t& desc, hipStream_t stream);
hipError_t launch_attn(const AttnArgs& a, hipStream_t stream);
// the kernel for 128 and more query rows per kv head (kvq_prefill.hip)
bool prefill_applies(const AttnArgs& a);
hipError_t launch_prefill(const AttnArgs& a, hipStream_t stream);
// the same kernel over a prefix all sequences share, rows of all sequences stacked; leaves
// partials for the reduce (a.shared_groups > 0, a.prefix_chunks >= 1)
bool prefix_applies(const AttnArgs& a);
hipError_t launch_prefix(const AttnArgs& a, hipStream_t stream);
#ifdef KVQ_PROFILE  // the measurement build's switches (include/kvq_prof.h)
void set_prefill_kernel(bool on);
void set_profile_events(hipEvent_t before, hipEvent_t after);
void set_read_ceiling(bool on);
void set_skip_reduce(bool on);
void set_wave_clock(unsigned long long* buf);
#endif
hipError_t launch_block_copy(const void* pool_cache, const float* pool_scales,
                             const kvq_cache_desc_t& desc, const int32_t* block_ids, int32_t num,
                             void* packed_cache, float* packed_scales, bool to_packed,
                             hipStream_t stream);
hipError_t launch_repack(const void* src, void* dst, const kvq_cache_desc_t& desc,
                         bool to_canonical, hipStream_t stream);

}  // namespace kvq
