// extern "C" entry points declared in include/kvq.h: host-side validation first (no HIP call
// is made for a bad argument), then the kernel launches on the caller's stream.
#include <math.h>
#include <stdlib.h>

#include <mutex>

#include "kvq_internal.h"
#ifdef KVQ_PROFILE
#include "../../include/kvq_prof.h"
#endif

namespace {

bool desc_ok(const kvq_cache_desc_t* d, int* err) {
  if (!d) { *err = KVQ_E_NULLPTR; return false; }
  if (d->mode != KVQ_INT8_TOKEN_HEAD && d->mode != KVQ_FP8E4M3_BLOCK_HEAD &&
      d->mode != KVQ_BF16_PLAIN && d->mode != KVQ_FP8E4M3_TENSOR &&
      d->mode != KVQ_INT4_TOKEN_HEAD && d->mode != KVQ_INT4_GROUP32) {
    *err = KVQ_E_BAD_MODE;
    return false;
  }
  const int bs = d->block_size;
  const bool bs_ok = bs >= 16 && bs <= 256 && (bs & (bs - 1)) == 0;
  if (d->num_blocks < 0 || !bs_ok || d->num_kv_heads <= 0 ||
      (d->head_dim != 64 && d->head_dim != 128) ||
      (kvq::is_int4(d->mode) && d->head_dim != 128)) {
    *err = KVQ_E_BAD_SHAPE;
    return false;
  }
  // a pool beyond 2^46 bytes (64 TiB) is not a real one, and sizes must not wrap
  const unsigned __int128 bytes = (unsigned __int128)d->num_blocks * 2 * (unsigned)d->num_kv_heads *
                                  (unsigned)bs * (unsigned)d->head_dim * 2;
  if (bytes > ((unsigned __int128)1 << 46)) {
    *err = KVQ_E_BAD_SHAPE;
    return false;
  }
  return true;
}

// Wavefronts the current GPU holds at once at two per SIMD: compute units x 4 SIMDs x 2 (2048
// on a whole MI355X; fewer under a partition mode or a CU mask).  Read once per device; where
// no device can be asked (a machine without a GPU, where only sizes and validation run) the
// whole chip's figure stands in.
constexpr int kMaxDevices = 64;
std::mutex g_device_mutex;
int g_resident_waves[kMaxDevices] = {};

int64_t auto_waves() {
  constexpr int64_t kWholeChip = 256 * 4 * 2;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return kWholeChip;
  std::lock_guard<std::mutex> lock(g_device_mutex);
  if (g_resident_waves[dev] == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        cus <= 0 || cus > 4096)
      return kWholeChip;
    g_resident_waves[dev] = cus * 4 * 2;
  }
  return g_resident_waves[dev];
}

// the KVQ_DEBUG checks (defined with their kernels further down)
bool debug_checks();
int debug_check_slots(const int64_t* slot_mapping, int32_t num_tokens, int64_t num_slots,
                      hipStream_t stream);

int ilog2(int x) {
  int s = 0;
  while ((1 << s) < x) ++s;
  return s;
}

// Everything the launch needs that depends only on host-side arguments.
bool make_plan(const kvq_cache_desc_t* d, int32_t batch, int32_t q_len, int32_t num_q_heads,
               int32_t max_seq_len, int32_t chunk_tokens, int32_t shared_prefix_tokens,
               kvq::AttnPlan* plan, int* err) {
  if (!desc_ok(d, err)) return false;
  if (batch < 0 || q_len < 1 || q_len > KVQ_MAX_Q_LEN || num_q_heads <= 0 ||
      num_q_heads % d->num_kv_heads != 0 || max_seq_len < 0 || chunk_tokens < 0 ||
      chunk_tokens % 64 != 0 || shared_prefix_tokens < 0) {
    *err = KVQ_E_BAD_SHAPE;
    return false;
  }
  const int group = num_q_heads / d->num_kv_heads;
  // (every product below is taken in a type that holds it: the arguments are only known to be
  // non-negative 32-bit numbers at this point)
  const int64_t rows = (int64_t)group * q_len;
  // (the group-scaled int4 kernels hold one accumulator per channel group: one row tile)
  const int64_t row_tiles = rows <= 16 || d->mode == KVQ_INT4_GROUP32 ? 1 : 2;
  const int64_t row_groups = (rows + 16 * row_tiles - 1) / (16 * row_tiles);
  const int64_t pairs = (int64_t)d->num_kv_heads * row_groups;
  // the flat list of 64-token groups can be no longer than this
  const unsigned __int128 flat_wide =
      (unsigned __int128)batch * (uint64_t)(((int64_t)max_seq_len + 63) / 64) * (uint64_t)pairs;
  if (rows > 0x7FFFFFFF || pairs > 0x7FFFFFFF || flat_wide > 0x7FFFFFFF) {
    *err = KVQ_E_BAD_SHAPE;
    return false;
  }
  const int64_t flat_max = (int64_t)flat_wide;
  plan->rows = (int32_t)rows;
  plan->row_tiles = (int32_t)row_tiles;
  plan->num_row_groups = (int32_t)row_groups;
  plan->pairs_per_seq = (int32_t)pairs;
  if (chunk_tokens == 0) {
    // even split over as many wavefronts as an MI355X keeps resident at this kernel's
    // register footprint: 256 CUs x 4 SIMDs x 2 (one 16-row tile, or two at head_dim 64) or
    // x 1 (two tiles at head_dim 128)
    // (an unquantized cache needs twice the registers per group: one wavefront per SIMD; so
    // does the group-scaled int4 cache, for its four accumulators per logit)
    const int64_t waves = auto_waves();
    const bool two_per_simd = (plan->row_tiles == 1 || d->head_dim == 64) &&
                              d->mode != KVQ_BF16_PLAIN && d->mode != KVQ_INT4_GROUP32;
    const int64_t resident = two_per_simd ? waves : waves / 2;
    plan->range_groups = 0;
    plan->num_waves = (int32_t)(flat_max < resident ? flat_max : resident);
  } else {
    plan->range_groups = chunk_tokens / 64;
    plan->num_waves = (int32_t)((flat_max + plan->range_groups - 1) / plan->range_groups);
  }
  if (plan->num_waves < 1) plan->num_waves = 1;
  // A shared prefix goes to the many-row kernel with all sequences' rows stacked, where that
  // kernel exists for the format, the call is not already its own (128 rows and more per kv
  // head), there is a second sequence to share with and the prefix fits the declared lengths.
  // It is cut into pieces so that about two workgroups per compute unit come about.
  plan->shared_groups = 0;
  plan->prefix_chunks = 1;
  const int64_t stacked = (int64_t)batch * rows;
  if (shared_prefix_tokens >= 64 && shared_prefix_tokens <= max_seq_len && batch >= 2 &&
      rows < 128 && d->mode != KVQ_INT4_GROUP32 && stacked <= (1 << 30)) {
    plan->shared_groups = shared_prefix_tokens / 64;
    const int64_t walks = d->num_kv_heads * ((stacked + 127) / 128);
    int64_t chunks = (auto_waves() / 4 + walks - 1) / walks;
    if (chunks > kvq::kMaxPrefixChunks) chunks = kvq::kMaxPrefixChunks;
    if (chunks > plan->shared_groups) chunks = plan->shared_groups;
    plan->prefix_chunks = (int32_t)chunks;
  }
  // one partial per (wavefront range, pair) crossing, numbered wave + pair index; behind them
  // one per (piece of the shared prefix, pair)
  const size_t slots =
      (size_t)plan->num_waves +
      (size_t)batch * plan->pairs_per_seq * (plan->shared_groups > 0 ? 1 + plan->prefix_chunks : 1);
  const size_t slot_rows = slots * 16 * plan->row_tiles;
  plan->acc_floats = slot_rows * d->head_dim;
  plan->ml_floats = slot_rows * 2;
  plan->prefix_ints = ((size_t)batch + 2 + 3) & ~(size_t)3;  // prefix sums, prefix length
  return true;
}

}  // namespace

extern "C" {

size_t kvq_cache_bytes(const kvq_cache_desc_t* desc) {
  int err;
  if (!desc_ok(desc, &err)) return 0;
  return (size_t)desc->num_blocks * 2 * desc->num_kv_heads * desc->block_size *
         kvq::row_bytes(desc->mode, desc->head_dim);
}

size_t kvq_scales_bytes(const kvq_cache_desc_t* desc) {
  int err;
  if (!desc_ok(desc, &err) || desc->mode == KVQ_BF16_PLAIN) return 0;
  if (desc->mode == KVQ_FP8E4M3_TENSOR) return 2 * sizeof(float);
  return (size_t)desc->num_blocks * sizeof(float) *
         kvq::block_scale_floats(desc->mode, desc->num_kv_heads, desc->block_size, desc->head_dim);
}

int kv_quant_write(const void* k, const void* v, const int64_t* slot_mapping,
                   int32_t num_tokens, void* cache, float* scales,
                   const kvq_cache_desc_t* desc, void* stream) {
  int err;
  if (!desc_ok(desc, &err)) return err;
  // one wavefront per (token, kv head, K|V) at most, four to a workgroup: the grid must fit
  if (num_tokens < 0 || (int64_t)num_tokens * desc->num_kv_heads * 2 / 4 > 0x7FFFFFFF)
    return KVQ_E_BAD_SHAPE;
  if (num_tokens == 0) return KVQ_OK;
  if (!k || !v || !slot_mapping || !cache) return KVQ_E_NULLPTR;
  if (!scales && desc->mode != KVQ_BF16_PLAIN) return KVQ_E_NULLPTR;
  if ((((uintptr_t)k | (uintptr_t)v | (uintptr_t)cache) & 15) != 0) return KVQ_E_BAD_SHAPE;
  if (debug_checks()) {
    const int rc = debug_check_slots(slot_mapping, num_tokens,
                                     (int64_t)desc->num_blocks * desc->block_size,
                                     (hipStream_t)stream);
    if (rc != KVQ_OK) return rc;
  }
  const hipError_t e = kvq::launch_write(k, v, slot_mapping, num_tokens, cache, scales, *desc,
                                         (hipStream_t)stream);
  return e == hipSuccess ? KVQ_OK : KVQ_E_HIP;
}

size_t paged_decode_attn_workspace_bytes(const kvq_cache_desc_t* desc, int32_t batch,
                                         int32_t q_len, int32_t num_q_heads,
                                         int32_t max_seq_len, int32_t chunk_tokens) {
  kvq::AttnPlan plan;
  int err;
  if (!make_plan(desc, batch, q_len, num_q_heads, max_seq_len, chunk_tokens, 0, &plan, &err))
    return 0;
  return (plan.acc_floats + plan.ml_floats + plan.prefix_ints) * sizeof(float);
}

size_t paged_decode_attn_prefix_workspace_bytes(const kvq_cache_desc_t* desc, int32_t batch,
                                                int32_t q_len, int32_t num_q_heads,
                                                int32_t max_seq_len, int32_t chunk_tokens,
                                                int32_t shared_prefix_tokens) {
  kvq::AttnPlan plan;
  int err;
  if (!make_plan(desc, batch, q_len, num_q_heads, max_seq_len, chunk_tokens, shared_prefix_tokens,
                 &plan, &err))
    return 0;
  return (plan.acc_floats + plan.ml_floats + plan.prefix_ints) * sizeof(float);
}

}  // extern "C"

// The scratch buffer of paged_decode_attn_static: device memory of the library's own, so that
// the call needs no workspace from a caller who cannot allocate one.  In host code this name is
// only a handle for hipGetSymbolAddress; the address kernels may use is looked up once per
// device (each device has its own copy at its own address).
static __device__ __align__(256) unsigned char scratch[KVQ_STATIC_WORKSPACE_BYTES];

namespace {

void* g_scratch_ptr[kMaxDevices] = {};  // per device, filled on the first call made there

// Device address of `scratch` on the current device (nullptr if the lookup fails).
void* scratch_on_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_device_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

// ---- KVQ_DEBUG=1 in the environment: the indices the kernels would follow blindly are checked
// on the device first.  A checking kernel runs ahead of the real one, the call waits for it
// (so a debug call synchronises with its stream and must not be made under graph capture), and
// an index out of range becomes KVQ_E_BAD_INDEX instead of a memory fault: nothing is trapped
// and the real kernel is not launched. ----
bool debug_checks() {
  const char* e = getenv("KVQ_DEBUG");
  return e && e[0] != '\0' && !(e[0] == '0' && e[1] == '\0');
}

__global__ void check_slots_kernel(const int64_t* __restrict__ slot_mapping, int32_t num_tokens,
                                   int64_t num_slots, int* __restrict__ word) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= num_tokens) return;
  if (slot_mapping[t] >= num_slots) {  // (negative = skip the token)
    atomicOr(&word[0], 1);
    atomicMin(&word[1], (int)t);
  }
}

// entry (b, j): sequence lengths inside [q_len, max_seq_len]; the table entries of every block
// below ceil(seq_lens[b] / block_size) inside [0, num_blocks); the first shared_blocks entries
// equal to sequence 0's (where both sequences are long enough for the prefix to be used)
__global__ void check_tables_kernel(const int32_t* __restrict__ block_tables,
                                    const int32_t* __restrict__ seq_lens, int32_t batch,
                                    int32_t max_blocks_per_seq, int32_t num_blocks,
                                    int32_t block_size, int32_t q_len, int32_t max_seq_len,
                                    int32_t shared_blocks, int32_t shared_tokens,
                                    int* __restrict__ word) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)batch * max_blocks_per_seq) return;
  const int b = (int)(i / max_blocks_per_seq), j = (int)(i - (int64_t)b * max_blocks_per_seq);
  const int L = seq_lens[b];
  if (L < q_len || L > max_seq_len) {
    if (j == 0) {
      atomicOr(&word[0], 2);
      atomicMin(&word[1], b);
    }
    return;
  }
  if (j >= (L + block_size - 1) / block_size) return;
  const int e = block_tables[i];
  if (e < 0 || e >= num_blocks) {
    atomicOr(&word[0], 4);
    atomicMin(&word[1], b);
  }
  if (j < shared_blocks && L >= shared_tokens && seq_lens[0] >= shared_tokens &&
      e != block_tables[j]) {
    atomicOr(&word[0], 8);
    atomicMin(&word[1], b);
  }
}

}  // namespace

static __device__ int debug_word[2];  // [0] what was found (bit set), [1] first token / sequence

namespace {

// Runs `launch_check(word)` on the stream and waits for its verdict.
template <class F>
int debug_verdict(hipStream_t stream, F launch_check) {
  int* word = nullptr;
  if (hipGetSymbolAddress((void**)&word, HIP_SYMBOL(debug_word)) != hipSuccess) return KVQ_E_HIP;
  const int init[2] = {0, 0x7FFFFFFF};
  int found[2] = {0, 0};
  if (hipMemcpyAsync(word, init, sizeof(init), hipMemcpyHostToDevice, stream) != hipSuccess)
    return KVQ_E_HIP;
  launch_check(word);
  if (hipGetLastError() != hipSuccess) return KVQ_E_HIP;
  if (hipMemcpyAsync(found, word, sizeof(found), hipMemcpyDeviceToHost, stream) != hipSuccess ||
      hipStreamSynchronize(stream) != hipSuccess)
    return KVQ_E_HIP;
  return found[0] ? KVQ_E_BAD_INDEX : KVQ_OK;
}

int debug_check_slots(const int64_t* slot_mapping, int32_t num_tokens, int64_t num_slots,
                      hipStream_t stream) {
  return debug_verdict(stream, [&](int* word) {
    hipLaunchKernelGGL(check_slots_kernel, dim3((unsigned)((num_tokens + 255) / 256)), dim3(256), 0,
                       stream, slot_mapping, num_tokens, num_slots, word);
  });
}

// Validation and launch shared by paged_decode_attn and paged_decode_attn_static.  With
// own_scratch the workspace is the library's static buffer, looked up only after every other
// check has passed (so that bad arguments are rejected without any HIP call).
int attn_call(const void* q, const void* cache, const float* scales,
              const kvq_cache_desc_t* desc, const int32_t* block_tables,
              int32_t max_blocks_per_seq, const int32_t* seq_lens, int32_t batch, int32_t q_len,
              int32_t num_q_heads, int32_t max_seq_len, float sm_scale, int32_t chunk_tokens,
              int32_t shared_prefix_tokens, float* out, void* workspace, size_t workspace_bytes,
              bool own_scratch, void* stream) {
  kvq::AttnPlan plan;
  int err;
  if (!make_plan(desc, batch, q_len, num_q_heads, max_seq_len, chunk_tokens, shared_prefix_tokens,
                 &plan, &err))
    return err;
  if (max_blocks_per_seq < 0 ||
      (int64_t)max_blocks_per_seq * desc->block_size < (int64_t)max_seq_len)
    return KVQ_E_BAD_SHAPE;
  if (batch == 0) return KVQ_OK;
  if (max_seq_len < q_len) return KVQ_E_BAD_SHAPE;
  if (!q || !cache || !block_tables || !seq_lens || !out) return KVQ_E_NULLPTR;
  if (!scales && desc->mode != KVQ_BF16_PLAIN) return KVQ_E_NULLPTR;
  // the kernels read q and the cache and write out in 16-byte pieces
  if ((((uintptr_t)q | (uintptr_t)cache | (uintptr_t)out) & 15) != 0) return KVQ_E_BAD_SHAPE;
  const size_t need = (plan.acc_floats + plan.ml_floats + plan.prefix_ints) * sizeof(float);
  if (own_scratch) {
    if (need > (size_t)KVQ_STATIC_WORKSPACE_BYTES) return KVQ_E_WORKSPACE;
    workspace = scratch_on_current_device();
    if (!workspace) return KVQ_E_HIP;
  } else if (need > 0) {
    if (!workspace) return KVQ_E_NULLPTR;
    if (workspace_bytes < need) return KVQ_E_WORKSPACE;
    if (((uintptr_t)workspace & 15) != 0) return KVQ_E_BAD_SHAPE;
  }

  if (debug_checks()) {
    const int64_t entries = (int64_t)batch * max_blocks_per_seq;
    if (entries > 0) {
      const int rc = debug_verdict((hipStream_t)stream, [&](int* word) {
        hipLaunchKernelGGL(check_tables_kernel, dim3((unsigned)((entries + 255) / 256)), dim3(256),
                           0, (hipStream_t)stream, block_tables, seq_lens, batch,
                           max_blocks_per_seq, desc->num_blocks, desc->block_size, q_len,
                           max_seq_len,
                           (plan.shared_groups * 64 + desc->block_size - 1) / desc->block_size,
                           plan.shared_groups * 64, word);
      });
      if (rc != KVQ_OK) return rc;
    }
  }

  kvq::AttnArgs a;
  a.q = (const uint16_t*)q;
  a.cache = (const uint8_t*)cache;
  a.scales = scales;
  a.block_tables = block_tables;
  a.seq_lens = seq_lens;
  a.out = out;
  a.ws_acc = (float*)workspace;
  a.ws_ml = (float*)workspace + plan.acc_floats;
  a.ws_prefix = (int32_t*)((float*)workspace + plan.acc_floats + plan.ml_floats);
  a.max_blocks_per_seq = max_blocks_per_seq;
  a.batch = batch;
  a.q_len = q_len;
  a.num_q_heads = num_q_heads;
  a.num_kv_heads = desc->num_kv_heads;
  a.group = num_q_heads / desc->num_kv_heads;
  a.rows = plan.rows;
  a.block_size = desc->block_size;
  a.bs_shift = ilog2(desc->block_size);
  a.head_dim = desc->head_dim;
  a.mode = desc->mode;
  a.row_tiles = plan.row_tiles;
  a.num_row_groups = plan.num_row_groups;
  a.pairs_per_seq = plan.pairs_per_seq;
  a.range_groups = plan.range_groups;
  a.num_waves = plan.num_waves;
  a.scale_log2 = sm_scale * 1.4426950408889634f;
  a.wave_clock = nullptr;
  a.shared_groups = plan.shared_groups;
  a.prefix_chunks = plan.prefix_chunks;
  const hipError_t e = kvq::launch_attn(a, (hipStream_t)stream);
  return e == hipSuccess ? KVQ_OK : KVQ_E_HIP;
}

}  // namespace

extern "C" {

int paged_decode_attn(const void* q, const void* cache, const float* scales,
                      const kvq_cache_desc_t* desc, const int32_t* block_tables,
                      int32_t max_blocks_per_seq, const int32_t* seq_lens, int32_t batch,
                      int32_t q_len, int32_t num_q_heads, int32_t max_seq_len, float sm_scale,
                      int32_t chunk_tokens, float* out, void* workspace,
                      size_t workspace_bytes, void* stream) {
  return attn_call(q, cache, scales, desc, block_tables, max_blocks_per_seq, seq_lens, batch,
                   q_len, num_q_heads, max_seq_len, sm_scale, chunk_tokens, 0, out, workspace,
                   workspace_bytes, false, stream);
}

int paged_decode_attn_prefix(const void* q, const void* cache, const float* scales,
                             const kvq_cache_desc_t* desc, const int32_t* block_tables,
                             int32_t max_blocks_per_seq, const int32_t* seq_lens, int32_t batch,
                             int32_t q_len, int32_t num_q_heads, int32_t max_seq_len,
                             float sm_scale, int32_t chunk_tokens, int32_t shared_prefix_tokens,
                             float* out, void* workspace, size_t workspace_bytes, void* stream) {
  return attn_call(q, cache, scales, desc, block_tables, max_blocks_per_seq, seq_lens, batch,
                   q_len, num_q_heads, max_seq_len, sm_scale, chunk_tokens, shared_prefix_tokens,
                   out, workspace, workspace_bytes, false, stream);
}

int paged_decode_attn_static(const void* q, const void* cache, const float* scales,
                             const kvq_cache_desc_t* desc, const int32_t* block_tables,
                             int32_t max_blocks_per_seq, const int32_t* seq_lens, int32_t batch,
                             int32_t q_len, int32_t num_q_heads, int32_t max_seq_len,
                             float sm_scale, int32_t chunk_tokens, float* out, void* stream) {
  return attn_call(q, cache, scales, desc, block_tables, max_blocks_per_seq, seq_lens, batch,
                   q_len, num_q_heads, max_seq_len, sm_scale, chunk_tokens, 0, out, nullptr, 0,
                   true, stream);
}

int kvq_cache_to_canonical(const void* cache, void* canonical, const kvq_cache_desc_t* desc,
                           void* stream) {
  int err;
  if (!desc_ok(desc, &err)) return err;
  if (kvq_cache_bytes(desc) == 0) return KVQ_OK;
  if (!cache || !canonical) return KVQ_E_NULLPTR;
  return kvq::launch_repack(cache, canonical, *desc, true, (hipStream_t)stream) == hipSuccess
             ? KVQ_OK
             : KVQ_E_HIP;
}

int kvq_cache_from_canonical(const void* canonical, void* cache, const kvq_cache_desc_t* desc,
                             void* stream) {
  int err;
  if (!desc_ok(desc, &err)) return err;
  if (kvq_cache_bytes(desc) == 0) return KVQ_OK;
  if (!cache || !canonical) return KVQ_E_NULLPTR;
  return kvq::launch_repack(canonical, cache, *desc, false, (hipStream_t)stream) == hipSuccess
             ? KVQ_OK
             : KVQ_E_HIP;
}

static int block_copy(const void* pool_cache, const float* pool_scales,
                      const kvq_cache_desc_t* desc, const int32_t* block_ids, int32_t num,
                      void* packed_cache, float* packed_scales, bool to_packed, void* stream) {
  int err;
  if (!desc_ok(desc, &err)) return err;
  // one workgroup per 4 KiB piece of a block; 32-bit byte offsets inside a block
  const int64_t block_bytes = (int64_t)2 * desc->num_kv_heads * desc->block_size *
                              kvq::row_bytes(desc->mode, desc->head_dim);
  if (num < 0 || block_bytes > 0x7FFFFFFF || (int64_t)num * ((block_bytes + 4095) / 4096) > 0x7FFFFFFF)
    return KVQ_E_BAD_SHAPE;
  if (num == 0) return KVQ_OK;
  if (!pool_cache || !block_ids || !packed_cache) return KVQ_E_NULLPTR;
  const bool block_scales = kvq::block_scale_floats(desc->mode, desc->num_kv_heads,
                                                    desc->block_size, desc->head_dim) != 0;
  if (block_scales && (!pool_scales || !packed_scales)) return KVQ_E_NULLPTR;
  if ((((uintptr_t)pool_cache | (uintptr_t)packed_cache) & 15) != 0) return KVQ_E_BAD_SHAPE;
  const hipError_t e = kvq::launch_block_copy(pool_cache, pool_scales, *desc, block_ids, num,
                                              packed_cache, packed_scales, to_packed,
                                              (hipStream_t)stream);
  return e == hipSuccess ? KVQ_OK : KVQ_E_HIP;
}

int kvq_blocks_export(const void* cache, const float* scales, const kvq_cache_desc_t* desc,
                      const int32_t* block_ids, int32_t num, void* packed_cache,
                      float* packed_scales, void* stream) {
  return block_copy(cache, scales, desc, block_ids, num, packed_cache, packed_scales, true, stream);
}

int kvq_blocks_import(const void* packed_cache, const float* packed_scales,
                      const kvq_cache_desc_t* desc, const int32_t* block_ids, int32_t num,
                      void* cache, float* scales, void* stream) {
  return block_copy(cache, scales, desc, block_ids, num, (void*)packed_cache,
                    (float*)packed_scales, false, stream);
}

#ifdef KVQ_PROFILE  // exported by the measurement build only (include/kvq_prof.h)
void kvq_profile_split_events(void* before, void* after) {
  kvq::set_profile_events((hipEvent_t)before, (hipEvent_t)after);
}

void kvq_profile_read_ceiling(int on) { kvq::set_read_ceiling(on != 0); }

void kvq_profile_skip_reduce(int on) { kvq::set_skip_reduce(on != 0); }
void kvq_profile_prefill_kernel(int on) { kvq::set_prefill_kernel(on != 0); }

void kvq_profile_wave_clock(void* buf) { kvq::set_wave_clock((unsigned long long*)buf); }
#endif

const char* kvq_strerror(int code) {
  switch (code) {
    case KVQ_OK: return "ok";
    case KVQ_E_NULLPTR: return "a required pointer is NULL";
    case KVQ_E_BAD_MODE: return "unknown quantization mode";
    case KVQ_E_BAD_SHAPE: return "unsupported shape or size argument";
    case KVQ_E_WORKSPACE: return "workspace too small";
    case KVQ_E_HIP: return "kernel launch failed";
    case KVQ_E_BAD_INDEX: return "slot, block-table entry or sequence length out of range (KVQ_DEBUG)";
    default: return "unknown error code";
  }
}

}  // extern "C"
