/*
 * kvq_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, fp64 CPU statement of what the quantized KV-cache write and the
 * quantized paged decode attention compute.  Only the tests, the smoke check and
 * the benchmark's CPU-baseline leg may load this library; the GPU library never
 * does and shares no source, header, table or helper with it.
 *
 * What it follows: the paper's KV-cache quantization passage (Section 7.2.2:
 * K and V are quantized on the fly from BF16 to INT8 / FP8 with dynamic scaling,
 * halving the cache), its description of the paged KV cache (Section 2: the cache
 * is a pool of fixed-size pages addressed through per-request tables) and of the
 * decode phase (Section 2: one new token attends over the whole stored history).
 * The paper fixes no constants; the ones used here (127, 448, round-half-even,
 * one scale per token per head for int8, one per block per head for fp8) are the
 * benchmark configurations' and are listed as readings in the design notes.
 *
 * Layout used by the oracle (the "canonical logical layout"):
 *   cache : u8  [num_blocks][2 (0=K,1=V)][num_kv_heads][block_size][head_dim]
 *           (mode 2: u16 bf16 bit patterns, same shape)
 *   scales: f32 [num_blocks][2][num_kv_heads][block_size]      (mode 0, int8)
 *           f32 [num_blocks][2][num_kv_heads]                  (mode 1, fp8)
 *           unused                                             (mode 2)
 *           f32 [2] (K, V), an input                           (mode 3)
 *           as mode 0                                          (mode 4; cache rows are
 *           head_dim / 2 bytes)
 *           f32 [num_blocks][2][num_kv_heads][block_size][head_dim / 32]  (mode 5; cache as
 *           mode 4)
 *   k, v, q : bf16 bit patterns (uint16), [tokens][heads][head_dim]
 *   out     : f64 [batch*q_len][num_q_heads][head_dim]
 *
 * No blocking, no online softmax, no split: the obvious loops.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_MODE_INT8 0
#define ORACLE_MODE_FP8 1
/* The unquantized cache the paper's Section 8.5 measures its quantized one against ("BF16
 * KV cache" baseline): the rows are stored as they are. */
#define ORACLE_MODE_BF16 2
/* "Per-tensor" scaling (Section 7.2.2) in its static form: one fp32 scale for all of a layer's
 * K and one for all of its V, fixed beforehand by the caller (scales[0], scales[1]); the write
 * only encodes, values beyond 448 scales saturate. */
#define ORACLE_MODE_FP8_TENSOR 3
/* INT4, the third format Section 7.2.2 names: codes in [-7, 7], one fp32 scale per (token,
 * kv head) as for int8 (scale = fp32 nearest to absmax / 7), two codes per byte: byte j of a
 * row holds channel 2j in its low nibble and channel 2j+1 in its high nibble, each a 4-bit
 * two's complement number.  The cache's last dimension is head_dim / 2 bytes. */
#define ORACLE_MODE_INT4 4
/* INT4 under "per-block dynamic scaling" (Section 7.2.2) with the block read as a group of
 * channels, the form int4 formats commonly take: one fp32 scale per (token, kv head, group of
 * 32 adjacent channels) = fp32 nearest to that group's absmax / 7; codes, nibble order and
 * cache shape as mode 4; scales f32 [num_blocks][2][num_kv_heads][block_size][head_dim / 32].
 * A channel with outliers then costs the resolution of its own group only. */
#define ORACLE_MODE_INT4_GROUP 5
#define ORACLE_INT4_GROUP 32

/* ---- O1: a bf16 bit pattern is the top half of an fp32; widening is exact ---- */
double oracle_bf16_to_f64(uint16_t bits) {
  uint32_t w = ((uint32_t)bits) << 16;
  float f;
  memcpy(&f, &w, sizeof f);
  return (double)f;
}

/* ---- OCP E4M3FN (Section 7.2.1/7.2.2 name "FP8"; the /448 constant selects this
 * flavour): 1 sign, 4 exponent (bias 7), 3 mantissa bits; no infinities; S.1111.111
 * is NaN; exponent field 0 is subnormal. ---- */
double oracle_fp8_decode(uint8_t code) {
  int sign = code >> 7, e = (code >> 3) & 15, m = code & 7;
  double mag;
  if (e == 15 && m == 7) return NAN;
  if (e == 0)
    mag = ldexp((double)m / 8.0, -6);
  else
    mag = ldexp(1.0 + (double)m / 8.0, e - 7);
  return sign ? -mag : mag;
}

/* Nearest representable value to the real y, ties to the even code (the even
 * mantissa), saturating at +-448 and never producing NaN; the sign bit is the sign
 * of y, kept even when the magnitude rounds to zero.  Written as a search over the
 * 127 finite magnitudes so that it is checkable by eye. */
uint8_t oracle_fp8_encode(double y) {
  static double magnitude[0x7F]; /* decode(0x00..0x7E), filled on first use */
  static int filled = 0;
  uint8_t sign = signbit(y) ? 0x80 : 0x00;
  double a = fabs(y);
  int best = 0;
  double best_err = INFINITY;
  if (!filled) {
    for (int c = 0; c <= 0x7E; ++c) magnitude[c] = oracle_fp8_decode((uint8_t)c);
    filled = 1;
  }
  if (isnan(y)) return 0x7F;
  if (a >= 448.0) return (uint8_t)(sign | 0x7E);
  for (int c = 0; c <= 0x7E; ++c) {
    double err = fabs(magnitude[c] - a);
    if (err < best_err || (err == best_err && (c & 1) == 0)) {
      best_err = err;
      best = c;
    }
  }
  return (uint8_t)(sign | best);
}

/* ---- int8: round-half-even of the exact quotient, clamped to [-127, 127].
 * x is a bf16 value and s an fp32 value, so the fp64 quotient is either exactly a
 * half-integer or at least 2^-25 away from one, far more than its 2^-53 relative
 * rounding error: rint() of it is the round-half-even of the exact quotient. ---- */
int8_t oracle_int8_encode(double x, float s) {
  double r;
  if (s == 0.0f) return 0;
  r = rint(x / (double)s); /* default rounding mode: to nearest, ties to even */
  if (r > 127.0) r = 127.0;
  if (r < -127.0) r = -127.0;
  return (int8_t)r;
}

/* int4: the same rule with 7 in place of 127 (the quotient of a bf16 by an fp32 value is a
 * half-integer exactly or at least 2^-25 away from one, whatever the divisor's size) */
int8_t oracle_int4_encode(double x, float s) {
  double r;
  if (s == 0.0f) return 0;
  r = rint(x / (double)s);
  if (r > 7.0) r = 7.0;
  if (r < -7.0) r = -7.0;
  return (int8_t)r;
}

/* scale = fp32 nearest to absmax / qmax */
float oracle_scale(double absmax, double qmax) { return (float)(absmax / qmax); }

static size_t tile_index(int64_t blk, int kv, int h, int H, int bs, int D) {
  return (((size_t)blk * 2 + (size_t)kv) * (size_t)H + (size_t)h) * (size_t)bs * (size_t)D;
}

/* ---- O2/O3: the write.  Returns 0, or -1 on a bad mode.
 * Tokens with a negative slot are skipped.
 * mode 0: every (token, head, K|V) row gets its own scale.
 * mode 1: all tokens of this call that land in one block form that block's "run";
 *   the block scale becomes max(previous scale, run absmax / 448), where the
 *   previous scale counts only if the run does not start at offset 0 of the block
 *   (a write at offset 0 declares the block fresh); if the scale grew, the codes
 *   already in the block below the run's first offset are re-expressed in the new
 *   scale. ---- */
int oracle_kv_quant_write(const uint16_t* k, const uint16_t* v, const int64_t* slot_mapping,
                          int32_t num_tokens, uint8_t* cache, float* scales, int32_t mode,
                          int32_t num_blocks, int32_t block_size, int32_t num_kv_heads,
                          int32_t head_dim) {
  const int H = num_kv_heads, D = head_dim, bs = block_size;
  (void)num_blocks;
  if (mode == ORACLE_MODE_INT8) {
    for (int32_t t = 0; t < num_tokens; ++t) {
      int64_t slot = slot_mapping[t];
      if (slot < 0) continue;
      int64_t blk = slot / bs;
      int off = (int)(slot % bs);
      for (int kv = 0; kv < 2; ++kv) {
        const uint16_t* src = kv ? v : k;
        for (int h = 0; h < H; ++h) {
          const uint16_t* row = src + ((size_t)t * H + h) * D;
          double m = 0.0;
          for (int d = 0; d < D; ++d) {
            double a = fabs(oracle_bf16_to_f64(row[d]));
            if (a > m) m = a;
          }
          float s = (m == 0.0) ? 0.0f : oracle_scale(m, 127.0);
          scales[(((size_t)blk * 2 + kv) * H + h) * bs + off] = s;
          uint8_t* dst = cache + tile_index(blk, kv, h, H, bs, D) + (size_t)off * D;
          for (int d = 0; d < D; ++d)
            dst[d] = (uint8_t)oracle_int8_encode(oracle_bf16_to_f64(row[d]), s);
        }
      }
    }
    return 0;
  }
  if (mode == ORACLE_MODE_BF16) {
    uint16_t* cache16 = (uint16_t*)cache;
    for (int32_t t = 0; t < num_tokens; ++t) {
      int64_t slot = slot_mapping[t];
      if (slot < 0) continue;
      int64_t blk = slot / bs;
      int off = (int)(slot % bs);
      for (int kv = 0; kv < 2; ++kv)
        for (int h = 0; h < H; ++h)
          memcpy(cache16 + tile_index(blk, kv, h, H, bs, D) + (size_t)off * D,
                 (kv ? v : k) + ((size_t)t * H + h) * D, sizeof(uint16_t) * (size_t)D);
    }
    return 0;
  }
  if (mode == ORACLE_MODE_INT4) {
    const int Db = D / 2; /* bytes per row */
    for (int32_t t = 0; t < num_tokens; ++t) {
      int64_t slot = slot_mapping[t];
      if (slot < 0) continue;
      int64_t blk = slot / bs;
      int off = (int)(slot % bs);
      for (int kv = 0; kv < 2; ++kv) {
        for (int h = 0; h < H; ++h) {
          const uint16_t* row = (kv ? v : k) + ((size_t)t * H + h) * D;
          double m = 0.0;
          for (int d = 0; d < D; ++d) {
            double a = fabs(oracle_bf16_to_f64(row[d]));
            if (a > m) m = a;
          }
          float s = (m == 0.0) ? 0.0f : oracle_scale(m, 7.0);
          scales[(((size_t)blk * 2 + kv) * H + h) * bs + off] = s;
          uint8_t* dst = cache + tile_index(blk, kv, h, H, bs, Db) + (size_t)off * Db;
          for (int j = 0; j < Db; ++j) {
            int lo = oracle_int4_encode(oracle_bf16_to_f64(row[2 * j]), s);
            int hi = oracle_int4_encode(oracle_bf16_to_f64(row[2 * j + 1]), s);
            dst[j] = (uint8_t)((lo & 15) | ((hi & 15) << 4));
          }
        }
      }
    }
    return 0;
  }
  if (mode == ORACLE_MODE_INT4_GROUP) {
    const int Db = D / 2, NG = D / ORACLE_INT4_GROUP;
    for (int32_t t = 0; t < num_tokens; ++t) {
      int64_t slot = slot_mapping[t];
      if (slot < 0) continue;
      int64_t blk = slot / bs;
      int off = (int)(slot % bs);
      for (int kv = 0; kv < 2; ++kv) {
        for (int h = 0; h < H; ++h) {
          const uint16_t* row = (kv ? v : k) + ((size_t)t * H + h) * D;
          uint8_t* dst = cache + tile_index(blk, kv, h, H, bs, Db) + (size_t)off * Db;
          float* sdst = scales + ((((size_t)blk * 2 + kv) * H + h) * bs + off) * NG;
          for (int g = 0; g < NG; ++g) {
            const uint16_t* grp = row + g * ORACLE_INT4_GROUP;
            double m = 0.0;
            for (int d = 0; d < ORACLE_INT4_GROUP; ++d) {
              double a = fabs(oracle_bf16_to_f64(grp[d]));
              if (a > m) m = a;
            }
            float s = (m == 0.0) ? 0.0f : oracle_scale(m, 7.0);
            sdst[g] = s;
            for (int j = 0; j < ORACLE_INT4_GROUP / 2; ++j) {
              int lo = oracle_int4_encode(oracle_bf16_to_f64(grp[2 * j]), s);
              int hi = oracle_int4_encode(oracle_bf16_to_f64(grp[2 * j + 1]), s);
              dst[g * (ORACLE_INT4_GROUP / 2) + j] = (uint8_t)((lo & 15) | ((hi & 15) << 4));
            }
          }
        }
      }
    }
    return 0;
  }
  if (mode == ORACLE_MODE_FP8_TENSOR) {
    for (int32_t t = 0; t < num_tokens; ++t) {
      int64_t slot = slot_mapping[t];
      if (slot < 0) continue;
      int64_t blk = slot / bs;
      int off = (int)(slot % bs);
      for (int kv = 0; kv < 2; ++kv) {
        const float s = scales[kv];
        for (int h = 0; h < H; ++h) {
          const uint16_t* row = (kv ? v : k) + ((size_t)t * H + h) * D;
          uint8_t* dst = cache + tile_index(blk, kv, h, H, bs, D) + (size_t)off * D;
          for (int d = 0; d < D; ++d)
            dst[d] = (s > 0.0f) ? oracle_fp8_encode(oracle_bf16_to_f64(row[d]) / (double)s) : 0x00;
        }
      }
    }
    return 0;
  }
  if (mode != ORACLE_MODE_FP8) return -1;

  /* mode 1: visit each touched block once, in order of first appearance. */
  char* done = (char*)calloc((size_t)(num_tokens > 0 ? num_tokens : 1), 1);
  int32_t* run = (int32_t*)malloc(sizeof(int32_t) * (size_t)(num_tokens > 0 ? num_tokens : 1));
  for (int32_t t0 = 0; t0 < num_tokens; ++t0) {
    if (done[t0] || slot_mapping[t0] < 0) continue;
    int64_t blk = slot_mapping[t0] / bs;
    /* the run: every token of this call whose slot lies in blk */
    int32_t run_len = 0;
    int o_min = bs;
    for (int32_t t = t0; t < num_tokens; ++t) {
      int64_t slot = slot_mapping[t];
      if (slot < 0 || slot / bs != blk) continue;
      done[t] = 1;
      run[run_len++] = t;
      int off = (int)(slot % bs);
      if (off < o_min) o_min = off;
    }
    for (int kv = 0; kv < 2; ++kv) {
      const uint16_t* src = kv ? v : k;
      for (int h = 0; h < H; ++h) {
        double m = 0.0;
        for (int32_t i = 0; i < run_len; ++i) {
          const uint16_t* row = src + ((size_t)run[i] * H + h) * D;
          for (int d = 0; d < D; ++d) {
            double a = fabs(oracle_bf16_to_f64(row[d]));
            if (a > m) m = a;
          }
        }
        float* sp = scales + ((size_t)blk * 2 + kv) * H + h;
        float s_prev = (o_min > 0) ? *sp : 0.0f;
        float s_cand = (m == 0.0) ? 0.0f : oracle_scale(m, 448.0);
        float s_new = (s_prev > s_cand) ? s_prev : s_cand;
        *sp = s_new;
        uint8_t* tile = cache + tile_index(blk, kv, h, H, bs, D);
        if (o_min > 0 && s_new > s_prev && s_prev > 0.0f) {
          for (int off = 0; off < o_min; ++off)
            for (int d = 0; d < D; ++d) {
              uint8_t c = tile[(size_t)off * D + d];
              double val = oracle_fp8_decode(c);
              if (isnan(val)) continue; /* NaN codes are left as they are */
              /* 4-bit x 24-bit product is exact in fp64; the quotient by a 24-bit
               * value is either exactly an e4m3 midpoint or >= 2^-29 (relative)
               * away from one, so its fp64 rounding cannot change the result. */
              tile[(size_t)off * D + d] = oracle_fp8_encode(val * (double)s_prev / (double)s_new);
            }
        }
        for (int32_t i = 0; i < run_len; ++i) {
          int off = (int)(slot_mapping[run[i]] % bs);
          const uint16_t* row = src + ((size_t)run[i] * H + h) * D;
          for (int d = 0; d < D; ++d) {
            uint8_t c = 0x00;
            if (s_new > 0.0f) c = oracle_fp8_encode(oracle_bf16_to_f64(row[d]) / (double)s_new);
            tile[(size_t)off * D + d] = c;
          }
        }
      }
    }
  }
  free(run);
  free(done);
  return 0;
}

/* ---- O4: dequantized value of logical element (blk, kv, h, off, d) ---- */
double oracle_dequant_at(const uint8_t* cache, const float* scales, int32_t mode, int64_t blk,
                         int kv, int h, int off, int d, int32_t block_size,
                         int32_t num_kv_heads, int32_t head_dim) {
  const int H = num_kv_heads, D = head_dim, bs = block_size;
  if (mode == ORACLE_MODE_INT4 || mode == ORACLE_MODE_INT4_GROUP) {
    uint8_t byte = cache[tile_index(blk, kv, h, H, bs, D / 2) + (size_t)off * (D / 2) + d / 2];
    int nib = (d & 1) ? (byte >> 4) : (byte & 15);
    int code = (nib ^ 8) - 8; /* 4-bit two's complement */
    size_t token = (((size_t)blk * 2 + kv) * H + h) * bs + off;
    if (mode == ORACLE_MODE_INT4) return (double)code * (double)scales[token];
    return (double)code *
           (double)scales[token * (D / ORACLE_INT4_GROUP) + d / ORACLE_INT4_GROUP];
  }
  if (mode == ORACLE_MODE_BF16)
    return oracle_bf16_to_f64(
        ((const uint16_t*)cache)[tile_index(blk, kv, h, H, bs, D) + (size_t)off * D + d]);
  uint8_t c = cache[tile_index(blk, kv, h, H, bs, D) + (size_t)off * D + d];
  if (mode == ORACLE_MODE_INT8) {
    double s = (double)scales[(((size_t)blk * 2 + kv) * H + h) * bs + off];
    return (double)(int8_t)c * s;
  }
  if (mode == ORACLE_MODE_FP8_TENSOR) return oracle_fp8_decode(c) * (double)scales[kv];
  return oracle_fp8_decode(c) * (double)scales[((size_t)blk * 2 + kv) * H + h];
}

/* Dequantize the first n positions of one sequence's K or V for one kv head into a
 * dense [n][head_dim] fp64 array, walking the block table. */
void oracle_gather_dequant(const uint8_t* cache, const float* scales, int32_t mode,
                           const int32_t* block_table_row, int32_t n, int kv, int h,
                           int32_t block_size, int32_t num_kv_heads, int32_t head_dim,
                           double* dense) {
  for (int32_t p = 0; p < n; ++p) {
    int64_t blk = block_table_row[p / block_size];
    int off = p % block_size;
    for (int d = 0; d < head_dim; ++d)
      dense[(size_t)p * head_dim + d] = oracle_dequant_at(cache, scales, mode, blk, kv, h, off, d,
                                                          block_size, num_kv_heads, head_dim);
  }
}

/* ---- O5: attention.  seq_lens[b] counts the q_len current tokens; query token j
 * of sequence b sees positions 0 .. seq_lens[b] - q_len + j (itself included).
 * q head hq reads kv head hq / (num_q_heads / num_kv_heads).
 * Returns 0, or -1 if some sequence is shorter than q_len. ---- */
int oracle_paged_decode_attn(const uint16_t* q, const uint8_t* cache, const float* scales,
                             int32_t mode, int32_t num_blocks, int32_t block_size,
                             int32_t num_kv_heads, int32_t head_dim, const int32_t* block_tables,
                             int32_t max_blocks_per_seq, const int32_t* seq_lens, int32_t batch,
                             int32_t q_len, int32_t num_q_heads, double sm_scale, double* out) {
  const int D = head_dim, G = num_q_heads / num_kv_heads;
  int bad = 0;
  (void)num_blocks;
  for (int32_t b = 0; b < batch; ++b)
    if (seq_lens[b] < q_len) bad = 1;
  if (bad) return -1;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int32_t b = 0; b < batch; ++b) {
    for (int32_t hq = 0; hq < num_q_heads; ++hq) {
      const int h = hq / G;
      const int32_t L = seq_lens[b];
      const int32_t* table = block_tables + (size_t)b * max_blocks_per_seq;
      double* z = (double*)malloc(sizeof(double) * (size_t)L);
      double* kd = (double*)malloc(sizeof(double) * (size_t)L * D);
      double* vd = (double*)malloc(sizeof(double) * (size_t)L * D);
      oracle_gather_dequant(cache, scales, mode, table, L, 0, h, block_size, num_kv_heads, D, kd);
      oracle_gather_dequant(cache, scales, mode, table, L, 1, h, block_size, num_kv_heads, D, vd);
      for (int32_t j = 0; j < q_len; ++j) {
        const int32_t n = L - q_len + j + 1;
        const uint16_t* qrow = q + (((size_t)b * q_len + j) * num_q_heads + hq) * D;
        double* orow = out + (((size_t)b * q_len + j) * num_q_heads + hq) * D;
        double zmax = -INFINITY, denom = 0.0;
        for (int32_t p = 0; p < n; ++p) {
          double dot = 0.0;
          for (int d = 0; d < D; ++d) dot += oracle_bf16_to_f64(qrow[d]) * kd[(size_t)p * D + d];
          z[p] = sm_scale * dot;
          if (z[p] > zmax) zmax = z[p];
        }
        for (int32_t p = 0; p < n; ++p) {
          z[p] = exp(z[p] - zmax);
          denom += z[p];
        }
        for (int d = 0; d < D; ++d) orow[d] = 0.0;
        for (int32_t p = 0; p < n; ++p) {
          double w = z[p] / denom;
          for (int d = 0; d < D; ++d) orow[d] += w * vd[(size_t)p * D + d];
        }
      }
      free(z);
      free(kd);
      free(vd);
    }
  }
  return 0;
}

/* The softmax weights alone, for one (sequence, query token, q head): w[0..n-1].
 * Same arithmetic as above; lets a test look at the weights. Returns n. */
int32_t oracle_attn_weights(const uint16_t* q, const uint8_t* cache, const float* scales,
                            int32_t mode, int32_t block_size, int32_t num_kv_heads,
                            int32_t head_dim, const int32_t* block_table_row, int32_t seq_len,
                            int32_t q_len, int32_t j, int32_t num_q_heads, int32_t hq,
                            int32_t q_token_index, double sm_scale, double* w) {
  const int D = head_dim, G = num_q_heads / num_kv_heads, h = hq / G;
  const int32_t n = seq_len - q_len + j + 1;
  const uint16_t* qrow = q + ((size_t)q_token_index * num_q_heads + hq) * D;
  double* kd = (double*)malloc(sizeof(double) * (size_t)n * D);
  double zmax = -INFINITY, denom = 0.0;
  oracle_gather_dequant(cache, scales, mode, block_table_row, n, 0, h, block_size, num_kv_heads, D,
                        kd);
  for (int32_t p = 0; p < n; ++p) {
    double dot = 0.0;
    for (int d = 0; d < D; ++d) dot += oracle_bf16_to_f64(qrow[d]) * kd[(size_t)p * D + d];
    w[p] = sm_scale * dot;
    if (w[p] > zmax) zmax = w[p];
  }
  for (int32_t p = 0; p < n; ++p) {
    w[p] = exp(w[p] - zmax);
    denom += w[p];
  }
  for (int32_t p = 0; p < n; ++p) w[p] /= denom;
  free(kd);
  return n;
}

int oracle_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp master
    n = omp_get_num_threads();
  }
#endif
  return n;
}
