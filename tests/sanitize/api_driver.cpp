// Driver for the sanitizer build of the library's host layer (tests/test_sanitizers.py):
// csrc/kvq_api.hip compiled for the host with -fsanitize=address,undefined, the kernel
// launchers of the other translation units replaced by the stubs below, so that everything the
// entry points do before a launch (validation, the split plan, workspace carving) runs under the
// sanitizers on a machine without a GPU.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "../../paper_2605_29639_amd/csrc/kvq_internal.h"

namespace kvq {
static int launches = 0;
static AttnArgs last;
hipError_t launch_write(const void*, const void*, const int64_t*, int32_t, void*, float*,
                        const kvq_cache_desc_t&, hipStream_t) { ++launches; return hipSuccess; }
hipError_t launch_attn(const AttnArgs& a, hipStream_t) { ++launches; last = a; return hipSuccess; }
hipError_t launch_block_copy(const void*, const float*, const kvq_cache_desc_t&, const int32_t*,
                             int32_t, void*, float*, bool, hipStream_t) { ++launches; return hipSuccess; }
hipError_t launch_repack(const void*, void*, const kvq_cache_desc_t&, bool, hipStream_t) {
  ++launches;
  return hipSuccess;
}
}  // namespace kvq

#define EXPECT(cond) do { if (!(cond)) { printf("failed: %s (line %d)\n", #cond, __LINE__); return 1; } } while (0)

int main() {
  void* fake = (void*)0x1000;
  const int modes[6] = {0, 1, 2, 3, 4, 5};
  for (int mode : modes) {
    for (int bs = 16; bs <= 256; bs *= 2) {
      kvq_cache_desc_t d = {mode, 1000, bs, 8, 128};
      EXPECT(kvq_cache_bytes(&d) > 0);
      EXPECT(kv_quant_write(fake, fake, (const int64_t*)fake, 5, fake, (float*)fake, &d, nullptr) == KVQ_OK);
      for (int q_len : {1, 4, 33, 1024}) {
        for (int chunk : {0, 64, 2048}) {
          const int batch = 7, Hq = 32, max_len = 4000, max_blocks = (max_len + bs - 1) / bs;
          const size_t need = paged_decode_attn_workspace_bytes(&d, batch, q_len, Hq, max_len, chunk);
          EXPECT(need > 0);
          // a workspace address the carved pointers can be checked against
          char* ws = (char*)0x100000;
          kvq::launches = 0;
          EXPECT(paged_decode_attn(fake, fake, (const float*)fake, &d, (const int32_t*)fake, max_blocks,
                                   (const int32_t*)fake, batch, q_len, Hq, max_len, 0.1f, chunk,
                                   (float*)fake, ws, need, nullptr) == KVQ_OK);
          EXPECT(kvq::launches == 1);
          const kvq::AttnArgs& a = kvq::last;
          EXPECT((char*)a.ws_acc == ws && (char*)a.ws_ml > ws && (char*)a.ws_prefix > (char*)a.ws_ml);
          EXPECT((char*)(a.ws_prefix + batch + 1) <= ws + need);
          EXPECT(a.num_waves >= 1 && a.pairs_per_seq == 8 * a.num_row_groups);
          EXPECT(mode != 5 || a.row_tiles == 1);
          EXPECT(paged_decode_attn(fake, fake, (const float*)fake, &d, (const int32_t*)fake, max_blocks,
                                   (const int32_t*)fake, batch, q_len, Hq, max_len, 0.1f, chunk,
                                   (float*)fake, ws, need - 1, nullptr) == KVQ_E_WORKSPACE);
        }
      }
    }
  }
  kvq_cache_desc_t absurd = {0, 1 << 30, 256, 1 << 20, 128};   // a pool of 2^66 bytes: rejected
  EXPECT(kvq_cache_bytes(&absurd) == 0 && kvq_scales_bytes(&absurd) == 0);
  kvq_cache_desc_t big = {0, 1 << 20, 256, 1 << 9, 128};       // 2^45 bytes: sizes beyond 32 bits
  EXPECT(kvq_cache_bytes(&big) == (size_t)1 << 45);
  EXPECT(paged_decode_attn_workspace_bytes(&big, 1 << 20, 1024, 1 << 20, 1 << 30, 0) == 0);
  EXPECT(paged_decode_attn_workspace_bytes(&big, 1 << 12, 8, 1 << 12, 1 << 14, 0) > ((size_t)1 << 32));
  EXPECT(kv_quant_write(fake, fake, (const int64_t*)fake, 2147483647, fake, (float*)fake, &big, nullptr) ==
         KVQ_E_BAD_SHAPE);
  EXPECT(kvq_blocks_export(fake, (const float*)fake, &big, (const int32_t*)fake, 1 << 30, fake,
                           (float*)fake, nullptr) == KVQ_E_BAD_SHAPE);
  puts("api sanitizer driver ok");
  return 0;
}
