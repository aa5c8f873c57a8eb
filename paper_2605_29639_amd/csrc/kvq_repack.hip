// Conversions between the library's physical cache (K in 4-token quads, V channel-major per
// 16-token sub-block, int8 codes in offset-binary form) and the canonical
// [block][K|V][head][token][channel] array of plain codes.  Not on the hot
// path: used to hand a cache to, or take one from, code that expects the canonical order.
#include "kvq_internal.h"

namespace kvq {
namespace {

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

}  // namespace

hipError_t launch_repack(const void* src, void* dst, const kvq_cache_desc_t& desc,
                         bool to_canonical, hipStream_t stream) {
  const size_t total = (size_t)desc.num_blocks * 2 * desc.num_kv_heads * desc.block_size *
                       desc.head_dim;
  if (total == 0) return hipSuccess;
  size_t blocks = (total + 255) / 256;
  if (blocks > 65536) blocks = 65536;
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
