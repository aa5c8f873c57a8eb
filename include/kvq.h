/*
 * kvq.h -- C ABI of the MI355X (gfx950) library for on-the-fly KV-cache quantization and
 * quantized paged decode attention.
 *
 * The operations are the ones the paper describes in its KV Cache Quantization passage
 * (Section 7.2.2: K and V are quantized from BF16 to INT8 or FP8 while generating, with
 * dynamic scaling, which halves the cache and relieves the decode phase's memory-bandwidth
 * pressure), on the paged KV cache of Section 2 (fixed-size blocks reached through
 * per-request block tables) and for the decode phase of Section 2 (each new token attends
 * over the whole stored history).  The paper fixes no constants; the ones below
 * (127, 448, round-half-to-even, scale granularity) are the benchmark configurations'.
 *
 * Conventions for every entry point
 *   - Every pointer marked "device" is GPU memory owned by the caller; the library
 *     allocates nothing, frees nothing and keeps no state between calls (the one exception,
 *     documented there, is the device address paged_decode_attn_static remembers).
 *   - Calls enqueue work on `stream` (a hipStream_t passed as void*; NULL = the default
 *     stream) and return at once: no host synchronisation, no device-to-host copy.
 *   - Return value: KVQ_OK (0) or a negative KVQ_E_* code.  Arguments are validated on the
 *     host before any HIP call, so a bad argument never launches anything.  Nothing is
 *     printed and no exception crosses the boundary.
 *   - Zero-size calls (num_tokens == 0, batch == 0) succeed without launching.
 *   - Not checked (the caller's contract): block ids and slots in range; no duplicate slot
 *     within one call; no NaN/Inf in k, v, q; |q| <= 65504; q_len <= seq_lens[b] <= max_seq_len;
 *     block-table entries valid for every block below ceil(seq_lens[b] / block_size).
 *   - With KVQ_DEBUG=1 in the environment (read at every call) kv_quant_write and
 *     paged_decode_attn first check on the device what they would otherwise follow blindly:
 *     slots below num_blocks * block_size; q_len <= seq_lens[b] <= max_seq_len; the table
 *     entries of every block in use inside [0, num_blocks).  A violation returns
 *     KVQ_E_BAD_INDEX and launches nothing else: no trap, no memory fault.  Such a call waits
 *     for its stream (it is a debugging aid: slower, and not for use under graph capture).
 */
#ifndef KVQ_H
#define KVQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Most query tokens per sequence in one paged_decode_attn call (1 in a decode step, a handful
 * when verifying speculated tokens, hundreds for a chunk of a prompt). */
#define KVQ_MAX_Q_LEN 1024

typedef enum {
  KVQ_INT8_TOKEN_HEAD = 0,    /* int8 codes in [-127,127], one fp32 scale per (token, kv head) */
  KVQ_FP8E4M3_BLOCK_HEAD = 1, /* OCP E4M3 (finite-only, max 448) codes, one fp32 scale per
                                 (cache block, kv head) */
  KVQ_BF16_PLAIN = 2,         /* no quantization: the bf16 rows as they are, no scales.  The
                                 baseline the paper's Section 8.5 measures its quantized
                                 cache against ("BF16 KV cache"); same entry points, twice
                                 the bytes */
  KVQ_FP8E4M3_TENSOR = 3,     /* E4M3 codes with static per-tensor scales: one fp32 scale for
                                 all of the layer's K, one for all of its V, chosen by the
                                 caller beforehand and only read by the library */
  KVQ_INT4_TOKEN_HEAD = 4,    /* int4 codes in [-7,7], two per byte, one fp32 scale per
                                 (token, kv head); head_dim 128 only */
  KVQ_INT4_GROUP32 = 5        /* the same codes and cache, one fp32 scale per (token, kv head,
                                 group of 32 adjacent channels): "per-block dynamic scaling"
                                 with a block of channels; head_dim 128 only */
} kvq_mode_t;

enum {
  KVQ_OK = 0,
  KVQ_E_NULLPTR = -1,    /* a required pointer is NULL */
  KVQ_E_BAD_MODE = -2,   /* desc->mode is not a kvq_mode_t */
  KVQ_E_BAD_SHAPE = -3,  /* unsupported head_dim / block_size / head counts / lengths */
  KVQ_E_WORKSPACE = -4,  /* workspace_bytes is smaller than paged_decode_attn_workspace_bytes() */
  KVQ_E_HIP = -5,        /* a kernel launch failed (hipGetLastError was not hipSuccess) */
  KVQ_E_BAD_INDEX = -6   /* only with KVQ_DEBUG=1: an index read on the device is out of range */
};

/* Shape of one layer's cache.  K and V of a layer live in one `cache` buffer and one
 * `scales` buffer.
 *
 * Logical element (blk, kv, h, off, d): block blk, kv = 0 for K / 1 for V, kv head h,
 * token offset off inside the block, channel d.  Physical byte position in `cache`:
 *     tile  = ((blk * 2 + kv) * num_kv_heads + h) * block_size * head_dim
 *     K:  tile + (off/4) * 4*head_dim + (d/16) * 64 + (off%4) * 16 + d%16
 *         (quads of 4 tokens; inside a quad: 16-channel slices x 4 tokens x 16 channels)
 *     V:  tile + (off/16) * 16*head_dim + d * 16 + off%16
 *         (sub-blocks of 16 tokens; inside one: channel-major rows of 16 tokens, the order
 *          the P.V matrix instruction consumes)
 * Both orders make the 16-byte piece one lane feeds to a matrix instruction contiguous and
 * let the four lanes of a quad read 64 contiguous bytes.  int8 codes are stored in
 * offset-binary form (stored byte = code XOR 0x80 = code + 128); e4m3 codes are stored as is.
 * kvq_cache_to_canonical / kvq_cache_from_canonical convert to and from the plain
 * [num_blocks][2][num_kv_heads][block_size][head_dim] order.
 * KVQ_BF16_PLAIN: 2-byte elements, tile = (...) * block_size * head_dim * 2 bytes and, in
 * elements inside a tile,
 *     K:  (off/4) * 4*head_dim + (d/8) * 32 + (off%4) * 8 + d%8
 *     V:  (off/16) * 16*head_dim + ((off%16)/8) * 8*head_dim + d * 8 + off%8
 * (the same idea with 8-element pieces); there is no scales buffer (its size is 0 and the
 * `scales` arguments are ignored and may be NULL).
 * KVQ_FP8E4M3_TENSOR: the cache is the e4m3 one; scales is f32 [2] = {K scale, V scale}.
 * KVQ_INT4_TOKEN_HEAD (head_dim 128): a tile is block_size * 64 bytes; a code is stored as the
 * nibble code + 8.  Eight codes that feed one lane of a matrix instruction share a 32-bit word,
 * element e of the eight in nibble e/2 (e even) or e/2 + 4 (e odd), so that one AND-OR
 * isolates two neighbouring elements as an f16 pair.  Word holding logical element (off, d):
 *     K:  (off/4) * 256 + ((d%32)/8) * 64 + (off%4) * 16 + (d/32) * 4,   e = d % 8
 *     V:  (off/16) * 1024 + (d/32) * 256 + (d%16) * 16 + ((d/16)%2) * 8 + ((off%16)/8) * 4,
 *         e = off % 8
 * scales as for KVQ_INT8_TOKEN_HEAD.  The canonical form packs channel 2j (low nibble) and
 * 2j+1 (high nibble) of a token in byte j, 4-bit two's complement, rows of head_dim/2 bytes.
 * KVQ_INT4_GROUP32: the cache of KVQ_INT4_TOKEN_HEAD; scales
 *         f32 [num_blocks][2][num_kv_heads][block_size][head_dim / 32].
 * scales: f32 [num_blocks][2][num_kv_heads][block_size]   for KVQ_INT8_TOKEN_HEAD
 *         f32 [num_blocks][2][num_kv_heads]               for KVQ_FP8E4M3_BLOCK_HEAD
 * Supported: head_dim 64 or 128; block_size a power of two in [16, 256]. */
typedef struct {
  int32_t mode;         /* kvq_mode_t */
  int32_t num_blocks;   /* physical blocks in the pool */
  int32_t block_size;   /* tokens per block */
  int32_t num_kv_heads;
  int32_t head_dim;
} kvq_cache_desc_t;

/* Buffer sizes in bytes for a descriptor (0 if the descriptor is invalid). Host only. */
size_t kvq_cache_bytes(const kvq_cache_desc_t* desc);
size_t kvq_scales_bytes(const kvq_cache_desc_t* desc);

/* Section 7.2.2, "On-the-fly Quantization": quantize num_tokens new K and V rows and store
 * them at their slots (slot = physical_block * block_size + offset; a negative slot skips
 * the token).
 *   k, v          device, bf16 [num_tokens][num_kv_heads][head_dim], read only, 16-byte aligned
 *   slot_mapping  device, int64 [num_tokens], read only
 *   cache, scales device, layouts above, updated in place; cache 16-byte aligned
 * Calls with at least 1024 tokens (a prompt) take kernels that handle 16 tokens per
 * wavefront; the result does not depend on which kernels run.
 * KVQ_INT8_TOKEN_HEAD: per (token, kv head), separately for K and V: scale = fp32 nearest to
 *   absmax/127 (0 for an all-zero row, whose codes are 0); code = round-half-even of the
 *   exact x/scale, clamped to [-127, 127].
 * KVQ_INT4_TOKEN_HEAD: as KVQ_INT8_TOKEN_HEAD with 7 in place of 127.
 * KVQ_INT4_GROUP32: the same per group of 32 adjacent channels: each group has its own absmax,
 *   scale and rounding.
 * KVQ_BF16_PLAIN: the rows are copied to their slots unchanged.
 * KVQ_FP8E4M3_TENSOR: code = encode(x / scales[kv]) (0x00 when the scale is 0), saturating at
 *   +-448; the scales are not modified.
 * KVQ_FP8E4M3_BLOCK_HEAD: the tokens of this call that fall into one block must be
 *   consecutive in token order with consecutive increasing slots (append order).  For each
 *   such run, per kv head, separately for K and V: s_prev = the stored block scale if the
 *   run starts above offset 0, else 0 (a write at offset 0 starts the block afresh);
 *   s_new = max(s_prev, fp32 nearest to run absmax/448) is stored; if s_new > s_prev > 0
 *   the codes already stored below the run's first offset are re-encoded as
 *   encode(decode(c) * s_prev / s_new); the new codes are encode(x / s_new) (0x00 when
 *   s_new == 0).  encode = nearest E4M3 value, ties to even, saturating at +-448.
 *   (Only this mode restricts the order of a call's tokens: a block's scale depends on all of
 *   the block's tokens.  Every other mode takes the tokens of a call in any order, with skipped
 *   tokens anywhere, as long as no slot appears twice.)
 * A block must not be written while another sequence's table references it. */
int kv_quant_write(const void* k, const void* v, const int64_t* slot_mapping,
                   int32_t num_tokens, void* cache, float* scales,
                   const kvq_cache_desc_t* desc, void* stream);

/* Bytes of device workspace paged_decode_attn needs for these arguments (split-K partial
 * results).  Host only; returns 0 on invalid arguments. */
size_t paged_decode_attn_workspace_bytes(const kvq_cache_desc_t* desc, int32_t batch,
                                         int32_t q_len, int32_t num_q_heads,
                                         int32_t max_seq_len, int32_t chunk_tokens);

/* Section 2, decode phase, over the quantized paged cache of Section 7.2.2: for sequence b,
 * query token j (0 <= j < q_len) and query head hq, attend over positions
 * 0 .. seq_lens[b] - q_len + j of kv head hq / (num_q_heads / num_kv_heads):
 *     out = sum_p softmax_p(sm_scale * q . Khat[p]) * Vhat[p],   Xhat = code * scale.
 * Position p lives at block_tables[b][p / block_size], offset p % block_size.
 * seq_lens[b] counts the q_len current tokens, which must already be in the cache.
 *   q             device, bf16 [batch*q_len][num_q_heads][head_dim], read only, 16-byte aligned
 *   block_tables  device, int32 [batch][max_blocks_per_seq], read only; entries past a
 *                 sequence's last block are never dereferenced
 *   seq_lens      device, int32 [batch], read only
 *   max_seq_len   host upper bound on seq_lens (sizes the launch grid)
 *   chunk_tokens  split-K granule: tokens of context per wavefront range, a multiple of 64;
 *                 0 = divide the work evenly over the wavefronts the GPU holds at once
 *   out           device, f32 [batch*q_len][num_q_heads][head_dim], written, 16-byte aligned
 *   workspace     device, >= paged_decode_attn_workspace_bytes(...) bytes, 16-byte aligned;
 *                 contents before and after the call are unspecified
 * Split-K: the 64-token groups of all (sequence, kv head) pairs form one flat list that is
 * cut into equal ranges, one per wavefront; a range that ends inside a pair leaves an
 * unnormalised partial (running max, sum, accumulator) in the workspace and a second kernel
 * merges a pair's partials by the log-sum-exp rule.  Results are deterministic run to run
 * (no atomics).
 * q_len is 1 in a decode step, a handful when speculated tokens are verified, and may be
 * hundreds for a chunk of a prompt attending over its quantized prefix and itself.  With 128
 * and more query rows per kv head ((num_q_heads / num_kv_heads) * q_len)
 * the call runs a kernel of its own that walks each (sequence, kv head) without a split and
 * dequantizes every K/V tile once for 128 rows (no workspace use, no second kernel); otherwise
 * the rows are taken 32 at a time, each such group streaming the keys and values again.  Either
 * way that use is bound by arithmetic, not by HBM.
 * Requires 1 <= q_len <= KVQ_MAX_Q_LEN and num_q_heads % num_kv_heads == 0. */
int paged_decode_attn(const void* q, const void* cache, const float* scales,
                      const kvq_cache_desc_t* desc, const int32_t* block_tables,
                      int32_t max_blocks_per_seq, const int32_t* seq_lens, int32_t batch,
                      int32_t q_len, int32_t num_q_heads, int32_t max_seq_len, float sm_scale,
                      int32_t chunk_tokens, float* out, void* workspace,
                      size_t workspace_bytes, void* stream);

/* paged_decode_attn for a batch whose sequences begin with the same blocks: a prompt prefix
 * served from the prefix cache, whose full blocks are shared by the requests that reuse it
 * (Section 1, "Intelligent KV Cache Management"; Section 5.2.3).
 *
 * shared_prefix_tokens is a promise: every block that holds a position below it is the same
 * physical block in every sequence's table (block_tables[b][i] == block_tables[0][i] for
 * those i).  The positions below floor(shared_prefix_tokens / 64) * 64 are then read once for
 * many sequences instead of once per sequence: a first kernel stacks the query rows of all
 * sequences, 128 to a workgroup, over the shared blocks (the many-row kernel of
 * paged_decode_attn, each K/V tile dequantized once per 128 rows) and leaves partials; the
 * streaming kernel covers the rest of each sequence; the reduce merges both.  The result is
 * paged_decode_attn's up to the order of the fp32 merges.  If the promise does not hold the
 * result is wrong, not undefined (every address still comes from a valid table entry); with
 * KVQ_DEBUG=1 it is checked and KVQ_E_BAD_INDEX returned.
 *
 * The prefix is used when every sequence has at least that many tokens (decided on the device
 * from seq_lens), for every format but KVQ_INT4_GROUP32, with batch >= 2 and fewer than 128
 * query rows per kv head; otherwise, and with shared_prefix_tokens < 64, the call is
 * paged_decode_attn.  shared_prefix_tokens < 0 is KVQ_E_BAD_SHAPE.
 *
 * workspace_bytes must be at least paged_decode_attn_prefix_workspace_bytes() for the same
 * arguments (more than paged_decode_attn needs: room for the first kernel's partials). */
size_t paged_decode_attn_prefix_workspace_bytes(const kvq_cache_desc_t* desc, int32_t batch,
                                                int32_t q_len, int32_t num_q_heads,
                                                int32_t max_seq_len, int32_t chunk_tokens,
                                                int32_t shared_prefix_tokens);
int paged_decode_attn_prefix(const void* q, const void* cache, const float* scales,
                             const kvq_cache_desc_t* desc, const int32_t* block_tables,
                             int32_t max_blocks_per_seq, const int32_t* seq_lens, int32_t batch,
                             int32_t q_len, int32_t num_q_heads, int32_t max_seq_len,
                             float sm_scale, int32_t chunk_tokens, int32_t shared_prefix_tokens,
                             float* out, void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, serving loops
 * and harnesses that forbid allocation): paged_decode_attn with the library's own scratch buffer
 * in place of the caller's workspace.  Same arguments otherwise, same kernels, same results.
 * The buffer is a static device array of KVQ_STATIC_WORKSPACE_BYTES that every GPU the library
 * runs on holds until the process ends; its device address is looked up on the first call made
 * on a device (a host-side lookup, not a stream operation; make that first call outside a
 * graph capture).  The call allocates and frees nothing.
 * Returns KVQ_E_WORKSPACE if paged_decode_attn_workspace_bytes() for these arguments exceeds
 * KVQ_STATIC_WORKSPACE_BYTES (the five benchmark configurations need 18 to 35 MB) and
 * KVQ_E_HIP if the buffer's address cannot be obtained.  All calls on one GPU share the one
 * buffer: calls that may overlap in time on one GPU (different streams, different threads) race
 * and must be serialised by the caller.  Nothing in it has to start at zero and its contents
 * after a call are unspecified. */
#define KVQ_STATIC_WORKSPACE_BYTES (64u << 20)
int paged_decode_attn_static(const void* q, const void* cache, const float* scales,
                             const kvq_cache_desc_t* desc, const int32_t* block_tables,
                             int32_t max_blocks_per_seq, const int32_t* seq_lens, int32_t batch,
                             int32_t q_len, int32_t num_q_heads, int32_t max_seq_len,
                             float sm_scale, int32_t chunk_tokens, float* out, void* stream);

/* Conversions between the physical cache above and the canonical
 * [num_blocks][2][num_kv_heads][block_size][head_dim] array of plain codes (int8 two's
 * complement / e4m3 bytes / bf16 bit patterns / int4 pairs); both device, kvq_cache_bytes()
 * long, must not overlap.  Used by tests and tools; not on the hot path. */
int kvq_cache_to_canonical(const void* cache, void* canonical, const kvq_cache_desc_t* desc,
                           void* stream);
int kvq_cache_from_canonical(const void* canonical, void* cache, const kvq_cache_desc_t* desc,
                             void* stream);

/* Block transfers between the pool and a packed staging area: the GPU end of the tiered
 * cache's LoadToGPU step (Section 3.3, Algorithm 1: blocks absent from GPU memory are loaded
 * from local CPU memory before the batch runs) and of its counterpart, the eviction of blocks
 * to CPU memory.  A block is one contiguous piece of `cache` (2 * num_kv_heads * block_size
 * * head_dim elements, in the physical order above) and one of `scales`, so the packed form
 * is simply those pieces one after another:
 *   kvq_blocks_export: packed block i  <-  pool block block_ids[i]
 *   kvq_blocks_import: pool block block_ids[i]  <-  packed block i
 *   block_ids      device, int32 [num], each in [0, num_blocks); for import, all different
 *   packed_cache   num * kvq_cache_bytes(desc) / num_blocks bytes, 16-byte aligned
 *   packed_scales  num * kvq_scales_bytes(desc) / num_blocks bytes (ignored for KVQ_BF16_PLAIN
 *                  and KVQ_FP8E4M3_TENSOR, whose scales are not part of a block)
 * The packed buffers may be device memory or pinned host memory that the GPU can address
 * (hipHostMalloc): the kernels then read or write it over the host link directly.
 * num == 0 succeeds without launching. */
int kvq_blocks_export(const void* cache, const float* scales, const kvq_cache_desc_t* desc,
                      const int32_t* block_ids, int32_t num, void* packed_cache,
                      float* packed_scales, void* stream);
int kvq_blocks_import(const void* packed_cache, const float* packed_scales,
                      const kvq_cache_desc_t* desc, const int32_t* block_ids, int32_t num,
                      void* cache, float* scales, void* stream);

/* Static, never-NULL description of a return code. */
const char* kvq_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* KVQ_H */
