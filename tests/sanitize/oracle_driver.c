/* Driver for the sanitizer build of the CPU checker (tests/test_sanitizers.py): every cache
 * mode, a ragged write with skipped tokens, an append that grows a block scale, attention with
 * several query tokens.  Buffers are heap allocations of exactly the documented sizes, so an
 * access outside them or any undefined arithmetic ends the run with a sanitizer report. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_kv_quant_write(const uint16_t* k, const uint16_t* v, const int64_t* slot_mapping,
                          int32_t num_tokens, uint8_t* cache, float* scales, int32_t mode,
                          int32_t num_blocks, int32_t block_size, int32_t num_kv_heads,
                          int32_t head_dim);
int oracle_paged_decode_attn(const uint16_t* q, const uint8_t* cache, const float* scales,
                             int32_t mode, int32_t num_blocks, int32_t block_size,
                             int32_t num_kv_heads, int32_t head_dim, const int32_t* block_tables,
                             int32_t max_blocks_per_seq, const int32_t* seq_lens, int32_t batch,
                             int32_t q_len, int32_t num_q_heads, double sm_scale, double* out);

static uint32_t rng_state = 12345u;
static uint16_t random_bf16(void) { /* a finite bf16 of moderate magnitude */
  rng_state = rng_state * 1664525u + 1013904223u;
  uint32_t sign = (rng_state >> 31) << 15, exp = 120u + ((rng_state >> 20) & 15u);
  return (uint16_t)(sign | (exp << 7) | ((rng_state >> 8) & 0x7Fu));
}

int main(void) {
  enum { NBLK = 6, BS = 16, H = 2, D = 128, HQ = 4, B = 2, QL = 2, MAXB = 3 };
  const int32_t lens[B] = {37, 19};
  const int32_t tables[B][MAXB] = {{4, 1, 5}, {2, 0, -1}};
  double checksum = 0.0;
  for (int mode = 0; mode <= 5; ++mode) {
    const size_t row = mode >= 4 ? D / 2 : D, esz = mode == 2 ? 2 : 1;
    const size_t cache_bytes = (size_t)NBLK * 2 * H * BS * row * esz;
    const size_t nscales = mode == 2 ? 0 : mode == 3 ? 2 : mode == 1 ? (size_t)NBLK * 2 * H
                           : mode == 5 ? (size_t)NBLK * 2 * H * BS * (D / 32)
                                       : (size_t)NBLK * 2 * H * BS;
    uint8_t* cache = calloc(cache_bytes, 1);
    float* scales = calloc(nscales ? nscales : 1, sizeof(float));
    if (mode == 3) { scales[0] = 0.05f; scales[1] = 0.02f; }
    for (int b = 0; b < B; ++b) {
      /* all but the last token in one call (one token skipped, outside fp8's run rule: at a
       * run's end), then the last token appended with 8x the magnitude */
      const int n = lens[b] - 1;
      uint16_t* k = malloc((size_t)lens[b] * H * D * 2);
      uint16_t* v = malloc((size_t)lens[b] * H * D * 2);
      int64_t* slots = malloc((size_t)lens[b] * 8);
      for (size_t i = 0; i < (size_t)lens[b] * H * D; ++i) { k[i] = random_bf16(); v[i] = random_bf16(); }
      memset(k + 3 * H * D, 0, (size_t)D * 2);                      /* an all-zero row */
      for (int p = 0; p < lens[b]; ++p) slots[p] = (int64_t)tables[b][p / BS] * BS + p % BS;
      const int64_t kept = slots[15];
      slots[15] = -1;
      if (oracle_kv_quant_write(k, v, slots, n, cache, scales, mode, NBLK, BS, H, D)) return 2;
      slots[15] = kept;
      if (oracle_kv_quant_write(k + 15 * H * D, v + 15 * H * D, slots + 15, 1, cache, scales, mode,
                                NBLK, BS, H, D)) return 3;
      for (size_t i = (size_t)n * H * D; i < (size_t)lens[b] * H * D; ++i) k[i] += 3u << 7, v[i] += 3u << 7;
      if (oracle_kv_quant_write(k + (size_t)n * H * D, v + (size_t)n * H * D, slots + n, 1, cache,
                                scales, mode, NBLK, BS, H, D)) return 4;
      free(k); free(v); free(slots);
    }
    uint16_t* q = malloc((size_t)B * QL * HQ * D * 2);
    for (size_t i = 0; i < (size_t)B * QL * HQ * D; ++i) q[i] = random_bf16();
    double* out = malloc((size_t)B * QL * HQ * D * sizeof(double));
    if (oracle_paged_decode_attn(q, cache, scales, mode, NBLK, BS, H, D, &tables[0][0], MAXB, lens,
                                 B, QL, HQ, 1.0 / sqrt((double)D), out)) return 5;
    for (size_t i = 0; i < (size_t)B * QL * HQ * D; ++i) {
      if (!isfinite(out[i])) return 6;
      checksum += out[i];
    }
    free(q); free(out); free(cache); free(scales);
  }
  printf("oracle sanitizer driver ok %.6f\n", checksum);
  return 0;
}
