// paged_decode_attn kernels (gfx950): decode attention (Section 2) over the quantized paged
// cache (Section 7.2.2).  Two launches: a streaming kernel that reads every K/V code from HBM
// once, and a small log-sum-exp reduce over the pieces a (sequence, kv head) was cut into.
//
// Work split.  All 64-token groups of all (sequence, kv head[, row group]) pairs form one flat
// list (sequence-major).  It is cut into equal ranges, one per wavefront (one wavefront = one
// workgroup), so every wavefront streams the same number of bytes whatever the mix of
// sequence lengths; a range that crosses from one pair into the next leaves a partial
// (max, sum, accumulator) for the pair it leaves.  A pair that lies inside one range is
// written to `out` directly.  Partial number (wave + pair index) is unique because ranges and
// pairs are both ordered cuts of the same list.
//
// Per wavefront and 64-token group (four 16-token sub-blocks):
//   * K codes: lane (m = lane%16, c = lane/16) loads 16-byte pieces of token
//     (sub-block m/4, token 4u + m%4) for u = 0..3, channels [64j + 16c, +16); the cache
//     keeps K in quads of 4 tokens so that the 4 lanes of a quad read 64 contiguous bytes.
//     That is directly the A operand (M = 16 tokens, K = 32 channels per instruction) of
//     v_mfma_f32_16x16x32_f16; q (f16) is the B operand with the G*q_len query rows that share
//     the kv head as the N columns.  The accumulator then holds, in lane
//     (row n = lane%16, g = lane/16), the logits of the 16 tokens of sub-block g.
//   * V codes are stored channel-major per 16-token sub-block, so lane (m, g) loads 16 bytes = 16 tokens of
//     sub-block g for channel 16t + m: the A operand (M = 16 channels, K = tokens) of the
//     P.V instruction, whose B operand is exactly the lane's own 16 probabilities.  No
//     shuffle, LDS transpose or re-layout sits between the two contractions.
//   * Codes become f16 exactly (int8, stored as code + 128: the byte is dropped into the
//     mantissa of 1024.0 and 1152 subtracted; e4m3: gfx950's packed fp8 -> f16 conversion), the
//     K scale multiplies the logit after the contraction and the V scale is folded into the
//     probability.
//   * Online softmax in base 2.  The running reference m is the maximum of
//     (logit + log2 V-scale), so the f16 probabilities p*sV stay in (0, 2^10] whatever the
//     magnitude of V; the plain softmax denominator is recovered as sum(P * 2^-lsv).
//   * Codes and scales are read exactly once, with non-temporal loads: streaming past the
//     caches measures ~6.9 TB/s on this machine against ~6.1 TB/s for ordinary loads.
//   * K and V each live in one register buffer: the next group's K codes are requested as
//     soon as QK^T has consumed the current ones, the next V codes as soon as P.V has.
#include "kvq_attn_common.h"

namespace kvq {
namespace {

// Position in the flat list of groups: sequence b, pair pr inside the sequence
// (pr = kv head * row groups + row group), group g of ng, sequence length L.  Wave-uniform.
struct Cursor {
  int b, pr, g, ng, L;
};

// Cross-lane scans and reductions on the DPP network (no LDS round trips): Hillis-Steele
// inside each row of 16 lanes (row_shr 1, 2, 4, 8), then the last lane of row 0 / row 2 into
// row 1 / row 3 (row_bcast:15) and lane 31 into rows 2 and 3 (row_bcast:31).  Lanes a step does
// not reach receive the operation's identity.  Lane 63 ends up holding the reduction.
template <class Op>
__device__ inline int dpp_scan_bits(int v, int identity, Op op) {
#define KVQ_DPP_STEP(CTRL, ROWS) \
  v = op(v, __builtin_amdgcn_update_dpp(identity, v, CTRL, ROWS, 0xF, false))
  KVQ_DPP_STEP(0x111, 0xF);  // row_shr:1
  KVQ_DPP_STEP(0x112, 0xF);  // row_shr:2
  KVQ_DPP_STEP(0x114, 0xF);  // row_shr:4
  KVQ_DPP_STEP(0x118, 0xF);  // row_shr:8
  KVQ_DPP_STEP(0x142, 0xA);  // row_bcast:15 into rows 1 and 3
  KVQ_DPP_STEP(0x143, 0xC);  // row_bcast:31 into rows 2 and 3
#undef KVQ_DPP_STEP
  return v;
}
__device__ inline int wave_incl_scan(int v) {
  return dpp_scan_bits(v, 0, [](int a, int b) { return a + b; });
}
__device__ inline int lane_value(int v, int lane_index) {  // lane_index wave-uniform
  return __builtin_amdgcn_readlane(v, lane_index);
}
__device__ inline float lane_value(float v, int lane_index) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane_index));
}
__device__ inline int wave_sum(int v) { return lane_value(wave_incl_scan(v), 63); }
__device__ inline int wave_min(int v) {
  return lane_value(dpp_scan_bits(v, 0x7FFFFFFF, [](int a, int b) { return a < b ? a : b; }), 63);
}
__device__ inline float wave_sum_f(float v) {
  const int r = dpp_scan_bits(__float_as_int(v), 0, [](int a, int b) {
    return __float_as_int(__int_as_float(a) + __int_as_float(b));
  });
  return __int_as_float(__builtin_amdgcn_readlane(r, 63));
}
__device__ inline float wave_max_f(float v) {
  const int r = dpp_scan_bits(__float_as_int(v), __float_as_int(-INFINITY), [](int a, int b) {
    return __float_as_int(fmaxf(__int_as_float(a), __int_as_float(b)));
  });
  return __int_as_float(__builtin_amdgcn_readlane(r, 63));
}

// How the flat list of `flat` groups is cut into wavefront ranges.  With a caller-given granule
// every range has `requested` groups; otherwise the list is cut into num_waves ranges whose
// sizes differ by at most one group, range w starting at floor(w * flat / num_waves), so that
// every compute unit, which holds the same number of wavefronts, streams the same number of
// bytes.  That floor is evaluated as w * q + floor(w * r / num_waves) with flat = q * num_waves
// + r: 32-bit arithmetic only (num_waves is below 2^16, so w * r is below 2^32).
struct Split {
  int requested, flat, num_waves, q, r;
};
__device__ inline Split make_split(int requested, int flat, int num_waves) {
  Split s;
  s.requested = requested;
  s.flat = flat;
  s.num_waves = num_waves;
  s.q = flat / num_waves;
  s.r = flat - s.q * num_waves;
  return s;
}
// First flat group of wavefront w's range (0 <= w <= num_waves).
__device__ inline int range_begin(const Split& s, int w) {
  if (s.requested > 0) return (int)min((long long)w * s.requested, (long long)s.flat);
  return w * s.q + (int)(((uint32_t)w * (uint32_t)s.r) / (uint32_t)s.num_waves);
}
// The wavefront whose range holds flat group f (0 <= f < flat): the w with
// range_begin(w) <= f < range_begin(w + 1), found from an estimate and at most a few steps.
__device__ inline int range_of(const Split& s, int f) {
  if (s.requested > 0) return f / s.requested;
  int w = (int)(((float)f + 0.5f) * ((float)s.num_waves / (float)s.flat));
  w = min(max(w, 0), s.num_waves - 1);
  while (range_begin(s, w) > f) --w;
  while (w + 1 < s.num_waves && range_begin(s, w + 1) <= f) ++w;
  return w;
}

// CEIL and CLOCK are false in the library proper; the measurement build (KVQ_PROFILE) also
// instantiates
//   CEIL = true: the read-ceiling twin, with the same ranges, addresses, load instructions and
//   pipeline, but the arithmetic replaced by an XOR of the loaded words (one dword per lane is
//   stored so that the loads stay);
//   CLOCK = true: the kernel itself, every wavefront also storing clock readings at fixed points.
// (The second launch bound, two wavefronts per SIMD, for the quantized one-tile kernels: they
// fit either way, but told so the compiler keeps everything in 200-224 VGPRs instead of parking
// values in AGPRs and copying them back, 1-2 % faster.  At head_dim 64 the two-tile kernels,
// double buffers included, fit 256 registers as well and run two per SIMD too.)
template <int MODE, int D, int NT, bool CEIL, int DEPTH, bool CLOCK>
__global__ __launch_bounds__(64, ((NT == 1 || D == 64) && MODE != KVQ_BF16_PLAIN && MODE != KVQ_INT4_GROUP32) ? 2 : 1) void
attn_stream_kernel(const AttnArgs p) {
  constexpr bool PLAIN = MODE == KVQ_BF16_PLAIN;  // unquantized cache: 2-byte elements
  // e4m3 codes, one scale per lane and group: the block's, or the whole layer's
  constexpr bool FP8 = MODE == KVQ_FP8E4M3_BLOCK_HEAD || MODE == KVQ_FP8E4M3_TENSOR;
  // int4 with one scale per (token, head, 32 channels): a matrix instruction contracts over
  // exactly one group of channels, so QK^T keeps one accumulator per group and the logit is
  // their sum weighted by the token's four K scales; P.V takes the probabilities times the V
  // scale of the group the channel tile belongs to (four versions of the B operand)
  constexpr bool GROUPED = MODE == KVQ_INT4_GROUP32;
  constexpr bool INT4 = MODE == KVQ_INT4_TOKEN_HEAD || GROUPED;  // two codes per byte (head_dim 128)
  // fp32 scales per token and head, K and V
  constexpr bool TOKEN_SCALE = MODE == KVQ_INT8_TOKEN_HEAD || INT4;
  static_assert(!GROUPED || (NT == 1 && D == 128), "group scales: one row tile, head_dim 128");
  constexpr int NG = GROUPED ? 4 : 1;  // scale groups per token
  using ScaleT = std::conditional_t<GROUPED, floatx4, float>;  // a token's K (or V) scales
  constexpr int EB = PLAIN ? 2 : 1;                // bytes per cache element
  constexpr int RB = INT4 ? D / 2 : D * EB;        // bytes per token row in a tile
  constexpr int DT = D / 16;
  constexpr int KJ = RB / 64;      // 16-byte K pieces per lane and quad
  constexpr int VW = RB / 16;      // 16-byte V pieces per lane
  constexpr int KS = D / 32;       // MFMA steps over the channels
  // matrix-instruction operand of 8 values: f16 (from codes) or the cache's own bf16
  using Operand = std::conditional_t<PLAIN, bf16x8, half8>;
  const int lane = threadIdx.x;
  const int m16 = lane & 15, g4 = lane >> 4;
  const int w = blockIdx.x;
  const int B = p.batch, Hp = p.pairs_per_seq;
  auto stamp = [&](int k, bool drain = false) {  // measurement build only
    if constexpr (CLOCK) {
      // slots 0..5 and 8..: shader clock; slots 6, 7: the constant 100 MHz clock at entry and
      // exit.  drain: first wait for every outstanding load, so that the reading marks the
      // arrival of what was requested so far.
      if (drain) __builtin_amdgcn_s_waitcnt(0);
      const unsigned long long t =
          (k == 6 || k == 7) ? __builtin_amdgcn_s_memrealtime() : __builtin_amdgcn_s_memtime();
      if (lane == 0) p.wave_clock[(size_t)w * 16 + k] = t;
    }
  };
  stamp(6);
  stamp(0);
  const int32_t* __restrict__ seq_lens = p.seq_lens;

  // ---- this wave's range [f0, f1) of the flat list, and where it starts ----
  // With a shared prefix the first P groups of every pair are the prefix kernel's (which reads
  // them once for many sequences), and the list holds groups P .. ng - 1 of every pair.  P is
  // the caller's figure if every sequence has that many full groups, else 0; the prefix kernel
  // takes the same decision from the same lengths.
  Cursor cur;
  int f0, f1;
  int P = 0;
  auto place = [&](int f, int base, int Li, int incl, int k0) {
    // among the sequences k0 + lane of this piece find the one that holds list position f;
    // base + incl = listed groups up to and including the lane's sequence
    const int i = k0 + lane;
    const int cnt = __popcll(__ballot(i < B && (base + incl) * Hp <= f));
    if (cnt == 64 || k0 + cnt >= B) return false;
    const int before = base + (cnt ? lane_value(incl, cnt - 1) : 0);
    cur.b = k0 + cnt;
    cur.L = lane_value(Li, cnt);
    cur.ng = (cur.L + 63) >> 6;
    const int len = cur.ng - P;  // the pair's groups in the list
    const int local = f - before * Hp;
    cur.pr = local / len;
    cur.g = P + (local - cur.pr * len);
    return true;
  };
  if (B <= 64) {
    // lane i holds sequence i: one load and one scan give the list's length, the prefix sums
    // the reduce wants and, by a ballot, the sequence this wave's range starts in
    const int Li = lane < B ? seq_lens[lane] : 0;
    const int ngi = (Li + 63) >> 6;
    const int incl = wave_incl_scan(ngi);
    if (p.shared_groups <= wave_min(lane < B ? Li >> 6 : 0x7FFFFFFF)) P = p.shared_groups;
    const int flat = (lane_value(incl, 63) - B * P) * Hp;
    if (!CEIL && w == 0) {
      if (lane < B) p.ws_prefix[lane + 1] = incl;
      if (lane == 0) {
        p.ws_prefix[0] = 0;
        p.ws_prefix[B + 1] = P;
      }
    }
    stamp(8, true);  // the sequence lengths have arrived
    const Split split = make_split(p.range_groups, flat, p.num_waves);
    f0 = range_begin(split, w);
    f1 = range_begin(split, w + 1);
    if (f0 >= f1) return;
    place(f0, 0, Li, incl - (lane + 1) * P, 0);
  } else {
    int total = 0, min_full = 0x7FFFFFFF;
    for (int k0 = 0; k0 < B; k0 += 64) {
      const int i = k0 + lane;
      const int Li = (i < B) ? seq_lens[i] : 0;
      total += (Li + 63) >> 6;
      if (i < B) min_full = min(min_full, Li >> 6);
    }
    if (p.shared_groups <= wave_min(min_full)) P = p.shared_groups;
    const int flat = (wave_sum(total) - B * P) * Hp;
    if (!CEIL && w == 0) {  // for the reduce: 64-token groups of the sequences before each one
      int base = 0;
      for (int k0 = 0; k0 < B; k0 += 64) {
        const int i = k0 + lane;
        const int incl = wave_incl_scan((i < B) ? (seq_lens[i] + 63) >> 6 : 0);
        if (i < B) p.ws_prefix[i + 1] = base + incl;
        base += lane_value(incl, 63);
      }
      if (lane == 0) {
        p.ws_prefix[0] = 0;
        p.ws_prefix[B + 1] = P;
      }
    }
    stamp(8, true);
    const Split split = make_split(p.range_groups, flat, p.num_waves);
    f0 = range_begin(split, w);
    f1 = range_begin(split, w + 1);
    if (f0 >= f1) return;
    int base = 0;
    for (int k0 = 0; k0 < B; k0 += 64) {
      const int i = k0 + lane;
      const int Li = (i < B) ? seq_lens[i] : 0;
      // (f0 lies inside the list, so the piece that holds its sequence is reached)
      const int incl = wave_incl_scan(i < B ? ((Li + 63) >> 6) - P : 0);
      if (place(f0, base, Li, incl, k0)) break;
      base += lane_value(incl, 63);
    }
  }
  stamp(9);  // the range and its first group are known
  auto advance = [&](Cursor& c) {  // the next group of the list
    if (++c.g < c.ng) return;
    c.g = P;
    if (++c.pr < Hp) return;
    c.pr = 0;
    do {  // (a sequence that is nothing but prefix has no groups in the list)
      ++c.b;
      c.L = (c.b < B) ? seq_lens[c.b] : 64 * (P + 1);
      c.ng = (c.L + 63) >> 6;
    } while (c.b < B && c.ng <= P);
  };

  if (CLOCK && lane == 0)  // slot 1: where the wavefront runs (XCC_ID << 32 | HW_ID)
    p.wave_clock[(size_t)w * 16 + 1] =
        ((unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 20) << 32) |
        (unsigned)__builtin_amdgcn_s_getreg((31 << 11) | 4);
  const int bs = p.block_size, bs_shift = p.bs_shift, H = p.num_kv_heads, NRG = p.num_row_groups;
  const uint8_t* __restrict__ cache = p.cache;
  const float* __restrict__ scales = p.scales;
  const uint32_t tile_bytes = (uint32_t)bs * RB;
  const int sbk = m16 >> 2;  // sub-block this lane reads K from
  const uint32_t block_stride = 2u * (uint32_t)H * tile_bytes;  // bytes per cache block
  const uint32_t k_lane = 64u * g4 + 16u * (m16 & 3);  // inside a 4-token quad
  const uint32_t v_lane = (uint32_t)H * tile_bytes + 16u * m16;  // inside a 16-token sub-block
  const uint32_t s_block_stride = TOKEN_SCALE                    ? 2u * H * bs * NG
                                  : (MODE == KVQ_FP8E4M3_TENSOR) ? 0u
                                                                 : 2u * H;
  const uint32_t s_kv = TOKEN_SCALE                    ? (uint32_t)H * bs * NG
                        : (MODE == KVQ_FP8E4M3_TENSOR) ? 1u
                                                       : (uint32_t)H;

  // block-table entries of the sub-blocks this lane reads K and V from
  auto fetch_entries = [&](const Cursor& c, int& blk_k, int& blk_v) {
    const int32_t* __restrict__ table = p.block_tables + (size_t)c.b * p.max_blocks_per_seq;
    const int pos0 = c.g << 6, last_sb = ((c.L - 1) >> 4) << 4;
    blk_k = table[min(pos0 + 16 * sbk, last_sb) >> bs_shift];
    blk_v = table[min(pos0 + 16 * g4, last_sb) >> bs_shift];
  };

  // K codes and both scales of a group; also works out where the group's V codes are
  auto load_k = [&](uintx4 (&kt)[4][KJ], ScaleT& sk, ScaleT& sv, const uint8_t*& vbase,
                    const Cursor& c, int blk_k, int blk_v) {
    const int pos0 = c.g << 6, last_sb = ((c.L - 1) >> 4) << 4;
    const uint32_t h = (uint32_t)(c.pr / NRG);
    const uint32_t off_k = (uint32_t)(min(pos0 + 16 * sbk, last_sb) & (bs - 1));
    const uint32_t off_v = (uint32_t)(min(pos0 + 16 * g4, last_sb) & (bs - 1));
    const uint8_t* kbase =
        cache + (size_t)blk_k * block_stride + (h * tile_bytes + off_k * RB + k_lane);
    vbase = cache + (size_t)blk_v * block_stride + (h * tile_bytes + v_lane + off_v * RB);
    const uint32_t s_lane = TOKEN_SCALE                    ? (h * bs + m16 + off_v) * NG
                            : (MODE == KVQ_FP8E4M3_TENSOR) ? 0u
                                                           : h;
    const ScaleT* sp = (const ScaleT*)(scales + (size_t)blk_v * s_block_stride + s_lane);
    constexpr uint32_t kSkip = GROUPED ? 4 : 1;  // floats per ScaleT
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int j = 0; j < KJ; ++j)
        kt[u][j] = __builtin_nontemporal_load((const uintx4*)(kbase + u * (4 * RB) + 256 * j));
    if constexpr (!PLAIN) {
      sk = __builtin_nontemporal_load(sp);
      sv = __builtin_nontemporal_load(sp + s_kv / kSkip);
    }
    if constexpr (PLAIN) {
      sk = 1.0f;
      sv = 1.0f;
    }
  };
  // (unquantized: piece 2 tt + half is channel tile tt, tokens 8 half .. 8 half + 7)
  auto load_v = [&](uintx4 (&vt)[VW], const uint8_t* vbase, const Cursor& c) {
#pragma unroll
    for (int x = 0; x < VW; ++x) {
      const int at = PLAIN ? (x & 1) * (16 * D) + 256 * (x >> 1) : 256 * x;
      vt[x] = __builtin_nontemporal_load((const uintx4*)(vbase + at));
    }
  };

  // ---- per-pair state: q as the B operand of QK^T, each row's causal length, the running
  // maximum / sum / accumulator ----
  Operand qb[NT][KS];
  [[maybe_unused]] floatx4 SG[GROUPED ? 3 : 1][4];  // group scales: contractions of groups 1..3
  [[maybe_unused]] half8 pbg[GROUPED ? 4 : 1][2];   // group scales: p x V scale, per group
  int nrow[NT];
  floatx4 acc[NT][DT];
  float m_run[NT], l_run[NT];
  uint32_t ceil_x = 0;
  auto begin_pair = [&](const Cursor& c) {
    if constexpr (CEIL) return;
    const int h = c.pr / NRG, rg = c.pr - h * NRG;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int r = (rg * NT + nt) * 16 + m16;
      const bool live = r < p.rows;
      const int j = live ? r / p.group : 0;
      const int gi = live ? r - j * p.group : 0;
      nrow[nt] = live ? c.L - p.q_len + j + 1 : c.L;
      const uint16_t* qrow =
          p.q + (((size_t)c.b * p.q_len + j) * p.num_q_heads + (size_t)h * p.group + gi) * D;
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        // the 8 channels this lane contributes to step s: the ones its K pieces hold
        const int d0 =
            PLAIN || INT4 ? 32 * s + 8 * g4 : 64 * (s >> 1) + 16 * g4 + 8 * (s & 1);
        const uintx4 raw = *(const uintx4*)(qrow + d0);
        if constexpr (PLAIN) {
          qb[nt][s] = __builtin_bit_cast(bf16x8, live ? raw : uintx4{0u, 0u, 0u, 0u});
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const _Float16 lo = (_Float16)__uint_as_float(raw[e] << 16);
            const _Float16 hi = (_Float16)__uint_as_float(raw[e] & 0xFFFF0000u);
            qb[nt][s][2 * e] = live ? lo : (_Float16)0.0f;
            qb[nt][s][2 * e + 1] = live ? hi : (_Float16)0.0f;
          }
        }
      }
      m_run[nt] = -INFINITY;
      l_run[nt] = 0.0f;
#pragma unroll
      for (int tt = 0; tt < DT; ++tt) acc[nt][tt] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
  };

  // leave a pair: final rows if this wave saw all of it, else a partial
  auto end_pair = [&](const Cursor& c, bool whole) {
    if constexpr (CEIL) return;
    const int h = c.pr / NRG, rg = c.pr - h * NRG;
    const size_t slot = (size_t)w + (size_t)c.b * Hp + c.pr;
    if (P > 0) whole = false;  // the pair's prefix is another partial, the prefix kernel's
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const float l = xor16_sum(l_run[nt]);
      const int rl = nt * 16 + m16;
      const int r = rg * NT * 16 + rl;
      if (r >= p.rows) continue;
      if (whole) {
        const int j = r / p.group, gi = r - j * p.group;
        float* orow =
            p.out + (((size_t)c.b * p.q_len + j) * p.num_q_heads + (size_t)h * p.group + gi) * D;
        const float inv = 1.0f / l;
#pragma unroll
        for (int tt = 0; tt < DT; ++tt) *(floatx4*)(orow + 16 * tt + 4 * g4) = acc[nt][tt] * inv;
      } else {
        const size_t row = slot * (NT * 16) + rl;
        float* arow = p.ws_acc + row * D;
#pragma unroll
        for (int tt = 0; tt < DT; ++tt) *(floatx4*)(arow + 16 * tt + 4 * g4) = acc[nt][tt];
        if (g4 == 0) {
          p.ws_ml[row * 2] = m_run[nt];
          p.ws_ml[row * 2 + 1] = l;
        }
      }
    }
  };

  // ---- S^T = K q^T ----
  auto qk = [&](const uintx4 (&kt)[4][KJ], floatx4 (&S)[NT][4]) {
    if constexpr (CEIL) {
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int j = 0; j < KJ; ++j) ceil_x ^= kt[u][j][0] ^ kt[u][j][1] ^ kt[u][j][2] ^ kt[u][j][3];
      return;
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int u = 0; u < 4; ++u) S[nt][u] = floatx4{0.f, 0.f, 0.f, 0.f};
    if constexpr (GROUPED) {
#pragma unroll
      for (int g = 0; g < 3; ++g)
#pragma unroll
        for (int u = 0; u < 4; ++u) SG[g][u] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int j = 0; j < KJ; ++j) {
        const uintx4 raw = kt[u][j];
        if constexpr (PLAIN) {
          const bf16x8 a = __builtin_bit_cast(bf16x8, raw);
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            S[nt][u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qb[nt][j], S[nt][u], 0, 0, 0);
        } else if constexpr (INT4) {  // word s of the piece: the 8 channels of step 4 j + s
#pragma unroll
          for (int st = 0; st < 4; ++st) {
            const half8 a = cvt_int4(raw[st]);
            if constexpr (GROUPED) {  // step st = channel group st: its own accumulator
              floatx4& dst = st == 0 ? S[0][u] : SG[st == 0 ? 0 : st - 1][u];
              dst = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, qb[0][st], dst, 0, 0, 0);
            } else {
#pragma unroll
              for (int nt = 0; nt < NT; ++nt)
                S[nt][u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, qb[nt][4 * j + st], S[nt][u], 0, 0, 0);
            }
          }
        } else {
          const half8 a0 = cvt8<MODE>(raw[0], raw[1]);
          const half8 a1 = cvt8<MODE>(raw[2], raw[3]);
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            S[nt][u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, qb[nt][2 * j], S[nt][u], 0, 0, 0);
            S[nt][u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, qb[nt][2 * j + 1], S[nt][u], 0, 0, 0);
          }
        }
      }
  };

  // ---- online softmax of a group: S (logits) -> pb (f16 probabilities x V scale); the body is
  // online_softmax in kvq_attn_common.h, shared with the many-row kernel.
  // TAIL = some row's causal length ends inside the group: positions past a row's length are
  // masked and scales of never-written slots are ignored. ----
  auto softmax_impl = [&](auto TAILC, floatx4 (&S)[NT][4], ScaleT sk, ScaleT sv, const Cursor& c,
                          Operand (&pb)[NT][2 * EB]) {
    constexpr bool TAIL = decltype(TAILC)::value;
    if constexpr (CEIL) {
      if constexpr (GROUPED) ceil_x ^= __float_as_uint(sk[0] + sk[1] + sk[2] + sk[3] + sv[0] + sv[1] + sv[2] + sv[3]);
      else ceil_x ^= __float_as_uint(sk) ^ __float_as_uint(sv);
      return;
    }
    const int pos0 = c.g << 6, L = c.L;
    if constexpr (GROUPED) {
#pragma clang fp contract(off)
      // a slot that was never written: its scales are not data
      const bool dead = TAIL && pos0 + 16 * g4 + m16 >= L;
      float skp[4], ratio[4];
      const float sv_max = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
      const float lsv = dead ? 0.0f : __builtin_amdgcn_logf(fmaxf(sv_max, kMinVScale));
      const float rsv = dead ? 0.0f : __builtin_amdgcn_exp2f(-lsv);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        skp[g] = dead ? 0.0f : sk[g] * p.scale_log2;
        ratio[g] = dead ? 0.0f : sv[g] * rsv;  // this group's V scale relative to the token's largest
      }
      // the logit: the four groups' contractions weighted by the token's four K scales
      static_for<16>([&](auto I) {
        constexpr int tix = decltype(I)::value, u = tix >> 2, i = tix & 3;
        float z = S[0][u][i] * row_bcast<tix>(skp[0]);
#pragma unroll
        for (int g = 1; g < 4; ++g) z = z + SG[g - 1][u][i] * row_bcast<tix>(skp[g]);
        S[0][u][i] = z;
      });
      online_softmax<MODE, NT, DT, TAIL>(S, 1.0f, lsv, rsv, pos0 + 16 * g4, nrow, m_run, l_run, acc, pb);
      // S now holds the probabilities times the largest V scale: one B operand per group
      static_for<16>([&](auto I) {
        constexpr int tix = decltype(I)::value, u = tix >> 2, i = tix & 3;
#pragma unroll
        for (int g = 0; g < 4; ++g)
          pbg[g][tix >> 3][tix & 7] = (_Float16)(S[0][u][i] * row_bcast<tix>(ratio[g]));
      });
    } else {
      // this lane's scales: logit factor, log2 of the V scale and its inverse
      float skp = sk * p.scale_log2;
      float lsv = PLAIN ? 0.0f : __builtin_amdgcn_logf(fmaxf(sv, kMinVScale));
      float rsv = PLAIN ? 1.0f : __builtin_amdgcn_exp2f(-lsv);
      if (TOKEN_SCALE && TAIL && pos0 + 16 * g4 + m16 >= L) {
        skp = 0.0f;  // a slot that was never written: its scales are not data
        lsv = 0.0f;
        rsv = 0.0f;
      }
      online_softmax<MODE, NT, DT, TAIL>(S, skp, lsv, rsv, pos0 + 16 * g4, nrow, m_run, l_run, acc, pb);
    }
  };
  auto softmax = [&](floatx4 (&S)[NT][4], ScaleT sk, ScaleT sv, const Cursor& c,
                     Operand (&pb)[NT][2 * EB]) {
    if ((c.g << 6) + 64 > c.L - p.q_len + 1)
      softmax_impl(std::true_type{}, S, sk, sv, c, pb);
    else
      softmax_impl(std::false_type{}, S, sk, sv, c, pb);
  };

  // ---- acc^T += V^T P^T ----
  // In a group that reaches past the sequence's last position the V bytes of the missing
  // tokens are whatever the pool holds; their probabilities are exactly 0, but an e4m3 NaN
  // code times 0 would still poison the sum, so those bytes are cleared first.
  auto pv_impl = [&](auto CLEARC, const uintx4 (&vt)[VW], const Operand (&pb)[NT][2 * EB],
                     const Cursor& c) {
    constexpr bool CLEAR = decltype(CLEARC)::value;
    if constexpr (CEIL) {
#pragma unroll
      for (int tt = 0; tt < VW; ++tt) ceil_x ^= vt[tt][0] ^ vt[tt][1] ^ vt[tt][2] ^ vt[tt][3];
      return;
    }
    if constexpr (PLAIN) {
      // a piece holds 8 tokens x 2 bytes: tokens 8 hf + 2 e and + 1 in word e
      const int live = c.L - ((c.g << 6) + 16 * g4);  // tokens of this lane's sub-block below L
#pragma unroll
      for (int x = 0; x < VW; ++x) {
        const int hf = x & 1, tt = x >> 1;
        uintx4 raw = vt[x];
        if constexpr (CLEAR) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int n = live - (8 * hf + 2 * e);
            raw[e] &= n >= 2 ? ~0u : n == 1 ? 0xFFFFu : 0u;
          }
        }
        const bf16x8 a = __builtin_bit_cast(bf16x8, raw);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          acc[nt][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pb[nt][hf], acc[nt][tt], 0, 0, 0);
          acc[nt][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pb[nt][2 + hf], acc[nt][tt], 0, 0, 0);
        }
      }
      return;
    }
    if constexpr (INT4) {
      // a piece holds two channel tiles (2 x and 2 x + 1): words 0, 1 the first tile's tokens
      // 0-7 and 8-15, words 2, 3 the second tile's
#pragma unroll
      for (int x = 0; x < VW; ++x)
#pragma unroll
        for (int par = 0; par < 2; ++par) {
          const half8 a0 = cvt_int4(vt[x][2 * par]);
          const half8 a1 = cvt_int4(vt[x][2 * par + 1]);
          if constexpr (GROUPED) {  // piece x = channels 32 x .. 32 x + 31 = group x
            acc[0][2 * x + par] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, pbg[x][0], acc[0][2 * x + par], 0, 0, 0);
            acc[0][2 * x + par] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, pbg[x][1], acc[0][2 * x + par], 0, 0, 0);
          } else {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
              acc[nt][2 * x + par] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, pb[nt][0], acc[nt][2 * x + par], 0, 0, 0);
              acc[nt][2 * x + par] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, pb[nt][1], acc[nt][2 * x + par], 0, 0, 0);
            }
          }
        }
      return;
    }
    uint32_t keep[4] = {~0u, ~0u, ~0u, ~0u};
    if constexpr (CLEAR) {
      const int live = c.L - ((c.g << 6) + 16 * g4);  // tokens of this lane's sub-block below L
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int n = min(max(live - 4 * e, 0), 4);
        keep[e] = n == 4 ? ~0u : (1u << (8 * n)) - 1u;
      }
    }
#pragma unroll
    for (int tt = 0; tt < DT; ++tt) {
      uintx4 raw = vt[tt];
      if constexpr (CLEAR) {
#pragma unroll
        for (int e = 0; e < 4; ++e) raw[e] &= keep[e];
      }
      const half8 a0 = cvt8<MODE>(raw[0], raw[1]);
      const half8 a1 = cvt8<MODE>(raw[2], raw[3]);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        acc[nt][tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a0, pb[nt][0], acc[nt][tt], 0, 0, 0);
        acc[nt][tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a1, pb[nt][1], acc[nt][tt], 0, 0, 0);
      }
    }
  };
  auto pv = [&](const uintx4 (&vt)[VW], const Operand (&pb)[NT][2 * EB], const Cursor& c) {
    if ((FP8 || PLAIN) && (c.g << 6) + 64 > c.L)
      pv_impl(std::true_type{}, vt, pb, c);
    else
      pv_impl(std::false_type{}, vt, pb, c);
  };

  // ---- main loop over the range.  Three cursors: cur (being computed), nxt (its codes are
  // being loaded), nn (its block-table entries are being fetched).  The table entries of a
  // group are always requested before the code loads that follow them in program order, so
  // waiting for an entry never waits for code loads issued behind it. ----
  int blk_k, blk_v;
  floatx4 S[NT][4];
  Operand pb[NT][2 * EB];
  const int count = f1 - f0;
  Cursor nxt = cur;
  if (count > 1) advance(nxt);
  Cursor nn = nxt;
  bool from_start = cur.g == P;  // did this wave see the current pair from its first listed group
  if constexpr (DEPTH == 1) {
    uintx4 kt[4][KJ], vt[VW];
    ScaleT sk, sv;
    const uint8_t* vbase;
    {
      int bk0, bv0;
      fetch_entries(cur, bk0, bv0);
      fetch_entries(nxt, blk_k, blk_v);
      begin_pair(cur);  // q is requested ahead of the codes so that it is not queued behind them
      __builtin_amdgcn_sched_barrier(0);
      stamp(10, true);  // the first table entries (and q) have arrived
      load_k(kt, sk, sv, vbase, cur, bk0, bv0);
      load_v(vt, vbase, cur);
    }
    stamp(2);
    // Two wavefronts share a SIMD and the hardware serves the older one first, so left alone
    // one of them races ahead and the other finishes late on a half-empty machine.  Each
    // wavefront therefore lowers its own issue priority as it progresses through its range:
    // whichever lags is served first and the two stay abreast.
    __builtin_amdgcn_s_setprio(3);
    const int q1 = count / 4, q2 = count / 2, q3 = count - count / 4;
    for (int i = 0; i + 1 < count; ++i) {  // steady state: a next group exists
      if (i == q1) __builtin_amdgcn_s_setprio(2);
      if (i == q2) __builtin_amdgcn_s_setprio(1);
      if (i == q3) __builtin_amdgcn_s_setprio(0);
      qk(kt, S);
      const ScaleT sk_cur = sk, sv_cur = sv;
      load_k(kt, sk, sv, vbase, nxt, blk_k, blk_v);
      if (i + 2 < count) advance(nn);
      fetch_entries(nn, blk_k, blk_v);
      softmax(S, sk_cur, sv_cur, cur, pb);
      pv(vt, pb, cur);
      load_v(vt, vbase, nxt);
      if (nxt.g == P) {  // the next group opens another pair
        end_pair(cur, from_start);
        begin_pair(nxt);
        from_start = true;
      }
      cur = nxt;
      nxt = nn;
    }
    stamp(3);
    qk(kt, S);  // the range's last group: nothing left to request
    softmax(S, sk, sv, cur, pb);
    pv(vt, pb, cur);
    stamp(4);
  } else {
    // Two full register buffers (one wavefront per SIMD; the 512-register file holds both):
    // a group's codes are requested a whole group ahead of their use.  The steady loop is
    // unrolled by two so that the buffers and the table-entry registers swap roles without
    // copies, and every load in it is unconditional (a load under a usually-true condition
    // would make the compiler's wait counts as strict as if the load were never issued).
    uintx4 kta[4][KJ], vta[VW], ktb[4][KJ], vtb[VW];
    ScaleT ska, sva, skb, svb;
    const uint8_t* vbase;
    int tk0, tv0, tk1, tv1;  // table entries of the group after the one being loaded
    Cursor c1 = nxt, c2 = nxt, c3 = nxt;  // groups i+1, i+2, i+3 (clamped to the range's last)
    if (count > 2) advance(c2);
    c3 = c2;
    if (count > 3) advance(c3);
    fetch_entries(cur, tk0, tv0);
    fetch_entries(c1, tk1, tv1);
    begin_pair(cur);
    __builtin_amdgcn_sched_barrier(0);
    load_k(kta, ska, sva, vbase, cur, tk0, tv0);
    load_v(vta, vbase, cur);
    auto leave = [&](const Cursor& next) {  // after a group: does the next one open another pair
      if (next.g == P) {
        end_pair(cur, from_start);
        begin_pair(next);
        from_start = true;
      }
      cur = next;
    };
    int i = 0;
    for (; i + 2 < count; i += 2) {  // groups i, i+1, i+2 exist
      // buffer a holds group i; tk1/tv1 are the entries of group i+1
      fetch_entries(c2, tk0, tv0);
      load_k(ktb, skb, svb, vbase, c1, tk1, tv1);
      load_v(vtb, vbase, c1);
      qk(kta, S);
      softmax(S, ska, sva, cur, pb);
      pv(vta, pb, cur);
      leave(c1);
      // buffer b holds group i+1; tk0/tv0 are the entries of group i+2
      fetch_entries(c3, tk1, tv1);
      load_k(kta, ska, sva, vbase, c2, tk0, tv0);
      load_v(vta, vbase, c2);
      qk(ktb, S);
      softmax(S, skb, svb, cur, pb);
      pv(vtb, pb, cur);
      leave(c2);
      c1 = c3;
      if (i + 4 < count) advance(c3);
      c2 = c3;
      if (i + 5 < count) advance(c3);
    }
    // one or two groups are left; buffer a holds group i
    if (i + 1 < count) {
      load_k(ktb, skb, svb, vbase, c1, tk1, tv1);
      load_v(vtb, vbase, c1);
      qk(kta, S);
      softmax(S, ska, sva, cur, pb);
      pv(vta, pb, cur);
      leave(c1);
      qk(ktb, S);
      softmax(S, skb, svb, cur, pb);
      pv(vtb, pb, cur);
    } else {
      qk(kta, S);
      softmax(S, ska, sva, cur, pb);
      pv(vta, pb, cur);
    }
  }
  end_pair(cur, from_start && cur.g == cur.ng - 1);
  stamp(5);
  stamp(7);
  // (one dword per lane into the accumulator area, which holds at least 16 * D floats per
  // wavefront, so that the loads cannot be optimised away)
  if constexpr (CEIL) p.ws_acc[(size_t)w * 64 + lane] = __uint_as_float(ceil_x & 0x3FFFFFFFu);
}

// ---- log-sum-exp merge of a pair's partials: one wavefront per (sequence, query head) and
// slice of the sequence's query tokens (blockIdx.y; up to 64 slices, so a handful of tokens get
// a wavefront each), each lane owning D/64 channels.  The kernel is a chain of memory round
// trips behind a launch, so it is written to keep that chain short: where the pair lies in the
// flat list comes from the prefix sums the streaming kernel's first wavefront left in the
// workspace (one round trip; a scan of seq_lens in every one of these wavefronts would cost
// batch^2 * heads loads); which wavefront ranges cover it is 32-bit arithmetic; then the (max,
// sum) pairs of up to 64 covering ranges, one per lane, and the first eight ranges' accumulator
// rows are requested together (one more round trip for a pair cut into at most eight pieces);
// further rows follow eight at a time. ----
template <int D>
__global__ __launch_bounds__(64) void attn_reduce_kernel(const AttnArgs p) {
  constexpr int E = D / 64;
  constexpr int NB = 8;  // accumulator rows requested at once
  typedef float floatE __attribute__((ext_vector_type(E)));
  typedef float float2v __attribute__((ext_vector_type(2)));
  const int hq = blockIdx.x % p.num_q_heads;
  const int b = blockIdx.x / p.num_q_heads;
  const int lane = threadIdx.x;
  // where the sequence lies in the flat list: the prefix sums the streaming kernel left, and
  // the length P (in groups) of the shared prefix it left to the prefix kernel (0: none)
  const int before = p.ws_prefix[b], next = p.ws_prefix[b + 1], total = p.ws_prefix[p.batch];
  const int P = p.ws_prefix[p.batch + 1];
  const int Hp = p.pairs_per_seq;
  const int all_pairs = p.batch * Hp;
  const Split split = make_split(p.range_groups, (total - p.batch * P) * Hp, p.num_waves);
  const int rt = 16 * p.row_tiles;
  const int h = hq / p.group;
  const int ng = next - before;
  const int na = P > 0 ? p.prefix_chunks : 0;  // partials the prefix kernel left for this pair
  const float* __restrict__ ws_acc = p.ws_acc + lane * E;
  const float2v* __restrict__ ws_ml = (const float2v*)p.ws_ml;
  // a range between two non-empty ones can be empty only if the list is shorter than the grid
  const bool sparse = split.requested == 0 && split.q == 0;
  int rg_known = -1, wb = 0, nb = 0;
  // (the wavefront takes the query tokens j = y, y + Y, ... one after the other: their rows
  // mostly lie in one row group, whose place in the list is then worked out once)
  for (int j = blockIdx.y; j < p.q_len; j += gridDim.y) {
    const int r = j * p.group + (hq - h * p.group);
    const int rg = r / rt, rl = r - rg * rt;
    const int pr = h * p.num_row_groups + rg;
    const int pair = b * Hp + pr;
    // the wavefront ranges that cover the pair's listed groups
    if (rg != rg_known && ng > P) {
      const int start = (before - b * P) * Hp + pr * (ng - P);
      wb = range_of(split, start);
      nb = range_of(split, start + (ng - P) - 1) - wb + 1;
      rg_known = rg;
    }
    if (na == 0 && nb == 1) continue;  // the streaming kernel already wrote the final rows
    const int n = na + nb;
    // the e-th partial of the pair: the prefix kernel's (one per chunk of the prefix, in slots
    // behind the streaming kernel's), then one per covering wavefront range
    auto row_of = [&](int e) {
      const size_t slot = e < na ? (size_t)p.num_waves + (size_t)(e + 1) * all_pairs + pair
                                 : (size_t)(wb + (e - na)) + pair;
      return slot * rt + rl;
    };
    // its (max, sum), or (-inf, 0) past the last one and for a range that is empty and left
    // no partial
    auto max_sum = [&](int e) {
      const int w = wb + (e - na);
      const bool live =
          e < n && (e < na || !sparse || range_begin(split, w) < range_begin(split, w + 1));
      return live ? ws_ml[row_of(e)] : float2v{-INFINITY, 0.0f};
    };
    auto load_rows = [&](floatE (&a)[NB], int e0, int count) {
#pragma unroll
      for (int k = 0; k < NB; ++k)
        if (k < count) a[k] = *(const floatE*)(ws_acc + row_of(e0 + k) * D);
    };
    floatE a_first[NB];
    load_rows(a_first, 0, n);

    // pass 1: the maximum over all partials
    const float2v ml_first = max_sum(lane);
    float M = ml_first[0];
    for (int e0 = 64; e0 < n; e0 += 64) M = fmaxf(M, max_sum(e0 + lane)[0]);
    M = wave_max_f(M);

    // pass 2: weights, denominator and the weighted sum of the accumulators
    floatE num = {};
    float den = 0.0f;
    for (int e0 = 0; e0 < n; e0 += 64) {
      const float2v ml = e0 == 0 ? ml_first : max_sum(e0 + lane);
      const float wgt = __builtin_amdgcn_exp2f(ml[0] - M);  // 0 for an empty range
      den += wgt * ml[1];
      const int count = min(64, n - e0);
      for (int k0 = 0; k0 < count; k0 += NB) {
        floatE a[NB];
        if (e0 == 0 && k0 == 0) {
#pragma unroll
          for (int k = 0; k < NB; ++k) a[k] = a_first[k];
        } else {
          load_rows(a, e0 + k0, count - k0);
        }
#pragma unroll
        for (int k = 0; k < NB; ++k) {
          if (k0 + k >= count) break;
          const float wk = lane_value(wgt, k0 + k);
          // (an empty range's row was never written: it must not enter even with weight 0)
          if (wk != 0.0f) num += wk * a[k];
        }
      }
    }
    den = wave_sum_f(den);
    float* o = p.out + (((size_t)b * p.q_len + j) * p.num_q_heads + hq) * D + lane * E;
    *(floatE*)o = num * (1.0f / den);
  }
}

#ifdef KVQ_PROFILE
// Measurement build only (libkvq_prof.so): events recorded around the streaming kernel, the
// read-ceiling twin or the clock-stamping variant in place of the kernel, the reduce skipped,
// many-row calls kept on the streaming kernels.  Process-global, not thread-safe.
hipEvent_t g_ev_before = nullptr, g_ev_after = nullptr;
bool g_read_ceiling = false;
bool g_skip_reduce = false;
bool g_prefill_kernel = true;
unsigned long long* g_wave_clock = nullptr;
#endif

// one 16-row tile: two wavefronts per SIMD, single register buffers; two tiles: one
// wavefront per SIMD, so the loads are double-buffered instead
// (an unquantized cache has twice the bytes per group: no room for a second buffer)
template <int MODE, int D, bool CEIL, bool CLOCK>
void launch_variant(const AttnArgs& a, hipStream_t stream) {
  constexpr int kDepth = MODE == KVQ_BF16_PLAIN ? 1 : 2;
  if constexpr (MODE == KVQ_INT4_GROUP32) {  // (the plan gives this format one row tile always)
    hipLaunchKernelGGL((attn_stream_kernel<MODE, D, 1, CEIL, 1, CLOCK>), dim3(a.num_waves), dim3(64), 0, stream, a);
  } else {
    if (a.row_tiles == 1)
      hipLaunchKernelGGL((attn_stream_kernel<MODE, D, 1, CEIL, 1, CLOCK>), dim3(a.num_waves), dim3(64), 0, stream, a);
    else
      hipLaunchKernelGGL((attn_stream_kernel<MODE, D, 2, CEIL, kDepth, CLOCK>), dim3(a.num_waves), dim3(64), 0, stream, a);
  }
}

template <int MODE, int D>
hipError_t launch_stream(const AttnArgs& a0, hipStream_t stream) {
#ifdef KVQ_PROFILE
  AttnArgs a = a0;
  a.wave_clock = g_wave_clock;
  // (with a shared prefix the first event lies before the prefix kernel)
  if (g_ev_before && (a.shared_groups == 0 || g_read_ceiling || g_skip_reduce))
    (void)hipEventRecord(g_ev_before, stream);
  if (g_read_ceiling)
    launch_variant<MODE, D, true, false>(a, stream);
  else if (g_wave_clock)
    launch_variant<MODE, D, false, true>(a, stream);
  else
    launch_variant<MODE, D, false, false>(a, stream);
  const hipError_t e = hipGetLastError();
  if (g_ev_after) (void)hipEventRecord(g_ev_after, stream);
  return e;
#else
  launch_variant<MODE, D, false, false>(a0, stream);
  return hipGetLastError();
#endif
}

}  // namespace

#ifdef KVQ_PROFILE
void set_profile_events(hipEvent_t before, hipEvent_t after) {
  g_ev_before = before;
  g_ev_after = after;
}
void set_read_ceiling(bool on) { g_read_ceiling = on; }
void set_skip_reduce(bool on) { g_skip_reduce = on; }
void set_prefill_kernel(bool on) { g_prefill_kernel = on; }
void set_wave_clock(unsigned long long* buf) { g_wave_clock = buf; }
#endif

hipError_t launch_attn(const AttnArgs& a, hipStream_t stream) {
#ifdef KVQ_PROFILE
  const bool stream_only = g_read_ceiling || g_skip_reduce;
  const bool many_rows_kernel = g_prefill_kernel && !g_read_ceiling;
#else
  constexpr bool stream_only = false, many_rows_kernel = true;
#endif
  if (many_rows_kernel && prefill_applies(a)) return launch_prefill(a, stream);
  hipError_t e;
  if (a.shared_groups > 0 && !stream_only) {  // the shared prefix, read once for many sequences
#ifdef KVQ_PROFILE
    if (g_ev_before) (void)hipEventRecord(g_ev_before, stream);
#endif
    e = launch_prefix(a, stream);
    if (e != hipSuccess) return e;
  }
  if (a.mode == KVQ_INT8_TOKEN_HEAD)
    e = a.head_dim == 128 ? launch_stream<KVQ_INT8_TOKEN_HEAD, 128>(a, stream)
                          : launch_stream<KVQ_INT8_TOKEN_HEAD, 64>(a, stream);
  else if (a.mode == KVQ_FP8E4M3_BLOCK_HEAD)
    e = a.head_dim == 128 ? launch_stream<KVQ_FP8E4M3_BLOCK_HEAD, 128>(a, stream)
                          : launch_stream<KVQ_FP8E4M3_BLOCK_HEAD, 64>(a, stream);
  else if (a.mode == KVQ_FP8E4M3_TENSOR)
    e = a.head_dim == 128 ? launch_stream<KVQ_FP8E4M3_TENSOR, 128>(a, stream)
                          : launch_stream<KVQ_FP8E4M3_TENSOR, 64>(a, stream);
  else if (a.mode == KVQ_INT4_TOKEN_HEAD)
    e = launch_stream<KVQ_INT4_TOKEN_HEAD, 128>(a, stream);  // (the only head_dim it takes)
  else if (a.mode == KVQ_INT4_GROUP32)
    e = launch_stream<KVQ_INT4_GROUP32, 128>(a, stream);
  else
    e = a.head_dim == 128 ? launch_stream<KVQ_BF16_PLAIN, 128>(a, stream)
                          : launch_stream<KVQ_BF16_PLAIN, 64>(a, stream);
  if (e != hipSuccess || stream_only) return e;
  // (a wavefront per (sequence, query head) and four query tokens, 64 per query head at most)
  const int per_head = (a.q_len + 3) / 4;
  const dim3 rgrid((unsigned)((size_t)a.batch * a.num_q_heads), (unsigned)(per_head < 64 ? per_head : 64));
  if (a.head_dim == 128)
    hipLaunchKernelGGL((attn_reduce_kernel<128>), rgrid, dim3(64), 0, stream, a);
  else
    hipLaunchKernelGGL((attn_reduce_kernel<64>), rgrid, dim3(64), 0, stream, a);
  return hipGetLastError();
}

}  // namespace kvq
