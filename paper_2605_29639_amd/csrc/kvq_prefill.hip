// paged_decode_attn for many query rows per kv head (a chunk of a prompt attending over its
// quantized prefix and itself, Section 2's prefill phase fed from the Section 7.2.2 cache).
//
// With 128 and more query rows per kv head the work is arithmetic, not memory traffic, and what
// has to be shared is the dequantization: the streaming kernel converts a group's codes once
// per 32 rows, this kernel once per 128.  A workgroup of four wavefronts owns 128 query rows of
// one (sequence, kv head) and walks the context from position 0 to the last position any of its
// rows may see (no split over the context, so no partials and no merge).  Per 64-token group
// each wavefront loads a quarter of the K and V codes, converts them to f16 and puts them in
// LDS in the order the matrix instruction wants its A operand (one 16-byte read per lane and
// instruction, no bank conflicts); after a barrier every wavefront runs QK^T, the online
// softmax and P.V for its own 32 rows against the shared operands.  LDS holds two groups, so
// one barrier per group suffices: while a group is consumed, the next one's codes are in
// flight and are converted into the other half.
//
// The arithmetic (logits in base 2 with the K scale applied after the contraction, V scale
// folded into the probability, f16 probabilities scaled by 2^10, masks) is the streaming
// kernel's, and so is the treatment of an unquantized cache: its bf16 rows are the operands
// as they are (copied to LDS, no conversion) and a probability enters P.V as two bf16 terms.
#include "kvq_attn_common.h"

namespace kvq {
namespace {

constexpr int kWavesPerGroup = 4;
constexpr int kRowsPerWorkgroup = kWavesPerGroup * 32;

// minimum over the wavefront
__device__ inline int wave_min_int(int v) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) v = min(v, __shfl_xor(v, d, 64));
  return v;
}

// PREFIX = true is the kernel for a prefix that every sequence of a decode or verification
// batch shares (the same physical blocks at the head of every block table; Section 1 and
// Section 5.2.3: prompt prefixes served from the prefix cache).  The query rows of all
// sequences are stacked, 128 to a workgroup, so a group of the prefix is read and converted
// once per 128 rows (four sequences of a 4-token verification step with 8 query heads per kv
// head) instead of once per sequence.  The prefix is cut into p.prefix_chunks pieces to get
// enough workgroups; a workgroup walks one piece and leaves, per row, an unnormalised partial
// (max, sum, accumulator) in the workspace, in the slots behind the streaming kernel's, which
// the reduce merges with the streaming kernel's partials over the rest of each sequence.
template <int MODE, int D, bool PREFIX>
__global__ __launch_bounds__(64 * kWavesPerGroup, 2) void attn_prefill_kernel(const AttnArgs p) {
  constexpr bool PLAIN = MODE == KVQ_BF16_PLAIN;  // unquantized cache: the operands are its bytes
  constexpr bool FP8 = MODE == KVQ_FP8E4M3_BLOCK_HEAD || MODE == KVQ_FP8E4M3_TENSOR;
  constexpr bool INT4 = MODE == KVQ_INT4_TOKEN_HEAD;  // two codes per byte (head_dim 128)
  constexpr bool TOKEN_SCALE = MODE == KVQ_INT8_TOKEN_HEAD || INT4;
  static_assert(!INT4 || D == 128, "int4 codes come with head_dim 128 only");
  constexpr int NT = 2;
  constexpr int EB = PLAIN ? 2 : 1;  // bytes per cache element
  constexpr int RB = INT4 ? D / 2 : D * EB;  // bytes per token row in a tile
  constexpr int DT = D / 16;       // 16-channel tiles of V / of the output
  constexpr int KJ = RB / 64;      // 16-byte K pieces per lane and quad
  constexpr int KS = D / 32;       // matrix-instruction steps over the channels
  constexpr int VT = DT / kWavesPerGroup;  // V tiles a wavefront converts
  constexpr int VP = INT4 ? VT / 2 : VT * EB;  // 16-byte V pieces per lane (int4: one piece = two tiles)
  // matrix-instruction operand of 8 values: f16 (from codes) or the cache's own bf16
  using Operand = std::conditional_t<PLAIN, bf16x8, half8>;
  __shared__ half8 k_ops[2][4][KS][64];    // [half][quad of the sub-block][step][lane]
  __shared__ half8 v_ops[2][DT][2][64];    // [half][channel tile][tokens 0-7 | 8-15][lane]
  __shared__ floatx4 s_ops[2][64];         // [half][token]: K scale * log2e / sqrt(D), log2 and
                                           // reciprocal of the V scale

  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int m16 = lane & 15, g4 = lane >> 4;
  const int H = p.num_kv_heads, G = p.group, bs = p.block_size, bs_shift = p.bs_shift;
  // rows a (kv head) has in this kernel: one sequence's, or all sequences' stacked
  const int all_rows = PREFIX ? p.batch * p.rows : p.rows;
  const int row_blocks = (all_rows + kRowsPerWorkgroup - 1) / kRowsPerWorkgroup;
  int P = 0;  // PREFIX: the shared groups, if every sequence has that many full ones
  if constexpr (PREFIX) {
    int min_full = 0x7FFFFFFF;
    for (int i = lane; i < p.batch; i += 64) min_full = min(min_full, p.seq_lens[i] >> 6);
    if (p.shared_groups > wave_min_int(min_full)) return;  // the streaming kernel does it all
    P = p.shared_groups;
  }
  // Workgroup -> (sequence, kv head, row block).  The hardware hands consecutive workgroups to
  // the eight XCDs in turn, each with an L2 of its own, and the row blocks of one (sequence,
  // kv head) read the same codes: they are placed on one XCD (workgroups x, x + 8, x + 16, ...)
  // so that the codes leave HBM once, not once per XCD.
  int pair, rb;  // PREFIX: pair = (piece of the prefix, kv head)
  {
    const int pairs = (PREFIX ? p.prefix_chunks : p.batch) * H, id = blockIdx.x;
    if (pairs % 8 == 0) {
      const int x = id & 7, k = id >> 3;
      pair = x + 8 * (k / row_blocks);
      rb = k % row_blocks;
    } else {
      pair = id / row_blocks;
      rb = id - pair * row_blocks;
    }
  }
  const int h = pair % H;
  // this wavefront's rows, and the groups [g0, ng) the workgroup has to walk
  const int r0 = rb * kRowsPerWorkgroup + wv * 32;
  const bool wave_live = r0 < all_rows;
  int b, L, g0, ng, n_min, chunk = 0;
  if constexpr (PREFIX) {
    chunk = pair / H;
    b = rb * kRowsPerWorkgroup / p.rows;  // whose block table: the first row's sequence (all agree)
    L = P << 6;                           // every position below it exists in every sequence
    g0 = (int)((long long)chunk * P / p.prefix_chunks);
    ng = (int)((long long)(chunk + 1) * P / p.prefix_chunks);
    n_min = 0;  // (set below, from the rows' own causal lengths)
  } else {
    b = pair / H;
    L = p.seq_lens[b];
    const int r_last = min(p.rows, (rb + 1) * kRowsPerWorkgroup) - 1;
    const int n_max = L - p.q_len + r_last / G + 1;
    g0 = 0;
    ng = (n_max + 63) >> 6;
    n_min = wave_live ? L - p.q_len + r0 / G + 1 : L;  // shortest causal length here
  }

  const uint8_t* __restrict__ cache = p.cache;
  const float* __restrict__ scales = p.scales;
  const int32_t* __restrict__ table = p.block_tables + (size_t)b * p.max_blocks_per_seq;
  const uint32_t tile_bytes = (uint32_t)bs * RB;
  const uint32_t block_stride = 2u * (uint32_t)H * tile_bytes;
  const int sbk = m16 >> 2;  // sub-block this lane reads K from
  const uint32_t k_lane = 64u * g4 + 16u * (m16 & 3) + (uint32_t)wv * (4 * RB);  // quad wv
  const uint32_t v_lane = (uint32_t)H * tile_bytes + 16u * m16 + 256u * (wv * (INT4 ? VP : VT));
  const uint32_t s_block_stride = TOKEN_SCALE ? 2u * H * bs : (MODE == KVQ_FP8E4M3_TENSOR ? 0u : 2u * H);
  const uint32_t s_kv = TOKEN_SCALE ? (uint32_t)H * bs : (MODE == KVQ_FP8E4M3_TENSOR ? 1u : (uint32_t)H);
  const int last_sb = ((L - 1) >> 4) << 4;

  // ---- q as the B operand of QK^T, causal lengths, running state ----
  Operand qb[NT][KS];
  int nrow[NT];
  floatx4 acc[NT][DT];
  float m_run[NT], l_run[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int rs = r0 + nt * 16 + m16;  // PREFIX: stacked row = sequence * rows + row
    const bool live = rs < all_rows;
    const int br = PREFIX ? (live ? rs / p.rows : 0) : b;
    const int r = PREFIX ? rs - br * p.rows : rs;
    const int j = live ? r / G : 0;
    const int gi = live ? r - j * G : 0;
    nrow[nt] = live ? (PREFIX ? p.seq_lens[br] : L) - p.q_len + j + 1 : L;
    const uint16_t* qrow =
        p.q + (((size_t)br * p.q_len + j) * p.num_q_heads + (size_t)h * G + gi) * D;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const int d0 = PLAIN || INT4 ? 32 * s + 8 * g4 : 64 * (s >> 1) + 16 * g4 + 8 * (s & 1);
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

  if constexpr (PREFIX) n_min = wave_min_int(min(nrow[0], nrow[1]));

  // ---- producer side: this wavefront's quarter of a group's codes ----
  struct Entries {
    int k, v;
  };
  auto fetch_entries = [&](int g, Entries& e) {  // g is clamped by the caller
    const int pos0 = g << 6;
    e.k = table[min(pos0 + 16 * sbk, last_sb) >> bs_shift];
    e.v = table[min(pos0 + 16 * g4, last_sb) >> bs_shift];
  };
  uintx4 rk[KJ], rv[VP];
  float sk_next = 0.0f, sv_next = 0.0f;
  auto issue_loads = [&](int g, const Entries& e) {
    const int pos0 = g << 6;
    const uint32_t off_k = (uint32_t)(min(pos0 + 16 * sbk, last_sb) & (bs - 1));
    const uint32_t off_v = (uint32_t)(min(pos0 + 16 * g4, last_sb) & (bs - 1));
    const uint8_t* kbase = cache + (size_t)e.k * block_stride + (h * tile_bytes + off_k * RB + k_lane);
    const uint8_t* vbase = cache + (size_t)e.v * block_stride + (h * tile_bytes + off_v * RB + v_lane);
#pragma unroll
    for (int j = 0; j < KJ; ++j) rk[j] = *(const uintx4*)(kbase + 256 * j);
    // (unquantized: piece 2 t + hf is channel tile t, tokens 8 hf .. 8 hf + 7)
#pragma unroll
    for (int x = 0; x < VP; ++x)
      rv[x] = *(const uintx4*)(vbase + (PLAIN ? (x & 1) * (16 * D) + 256 * (x >> 1) : 256 * x));
    if (!PLAIN && wv == 0) {  // the scales of the group's 64 tokens, lane = token
      const uint32_t s_lane = TOKEN_SCALE ? h * bs + m16 + off_v : (MODE == KVQ_FP8E4M3_TENSOR ? 0u : (uint32_t)h);
      const float* sp = scales + (size_t)e.v * s_block_stride + s_lane;
      sk_next = sp[0];
      sv_next = sp[s_kv];
    }
  };
  auto publish = [&](int g, int half) {  // convert the loaded codes and put them in LDS
    if constexpr (PLAIN) {  // bf16 rows are operands as they are; the LDS arrays hold their bits
#pragma unroll
      for (int j = 0; j < KJ; ++j) k_ops[half][wv][j][lane] = __builtin_bit_cast(half8, rk[j]);
      const int live = L - ((g << 6) + 16 * g4);  // tokens of this lane's sub-block below L
#pragma unroll
      for (int x = 0; x < VP; ++x) {
        uintx4 raw = rv[x];
        if ((g << 6) + 64 > L) {  // bf16 bit patterns of missing tokens: a NaN times 0 is NaN
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int n = live - (8 * (x & 1) + 2 * e);
            raw[e] &= n >= 2 ? ~0u : n == 1 ? 0xFFFFu : 0u;
          }
        }
        v_ops[half][wv * VT + (x >> 1)][x & 1][lane] = __builtin_bit_cast(half8, raw);
      }
      return;
    }
    if constexpr (INT4) {
      // K: word st of the lane's piece holds the 8 channels of step st; V: a piece holds two
      // channel tiles, words 0, 1 the first tile's tokens 0-7 and 8-15, words 2, 3 the second's
#pragma unroll
      for (int st = 0; st < 4; ++st) k_ops[half][wv][st][lane] = cvt_int4(rk[0][st]);
#pragma unroll
      for (int x = 0; x < VP; ++x)
#pragma unroll
        for (int w4 = 0; w4 < 4; ++w4)
          v_ops[half][2 * (wv * VP + x) + (w4 >> 1)][w4 & 1][lane] = cvt_int4(rv[x][w4]);
    } else {
#pragma unroll
      for (int j = 0; j < KJ; ++j) {
        k_ops[half][wv][2 * j][lane] = cvt8<MODE>(rk[j][0], rk[j][1]);
        k_ops[half][wv][2 * j + 1][lane] = cvt8<MODE>(rk[j][2], rk[j][3]);
      }
      uint32_t keep[4] = {~0u, ~0u, ~0u, ~0u};
      if (FP8 && (g << 6) + 64 > L) {  // V bytes of missing tokens: an e4m3 NaN times 0 is NaN
        const int live = L - ((g << 6) + 16 * g4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int n = min(max(live - 4 * e, 0), 4);
          keep[e] = n == 4 ? ~0u : (1u << (8 * n)) - 1u;
        }
      }
#pragma unroll
      for (int t = 0; t < VT; ++t) {
        uintx4 raw = rv[t];
#pragma unroll
        for (int e = 0; e < 4; ++e) raw[e] &= keep[e];
        v_ops[half][wv * VT + t][0][lane] = cvt8<MODE>(raw[0], raw[1]);
        v_ops[half][wv * VT + t][1][lane] = cvt8<MODE>(raw[2], raw[3]);
      }
    }
    // The scales go the same way: held in registers from the load to the softmax two iterations
    // later, they would have to be copied at the end of the iteration that requested them, and
    // that copy waits for the whole round trip to memory.
    if (wv == 0) {
      float skp = sk_next * p.scale_log2;
      float lsv = __builtin_amdgcn_logf(fmaxf(sv_next, kMinVScale));
      float rsv = __builtin_amdgcn_exp2f(-lsv);
      if (TOKEN_SCALE && (g << 6) + lane >= L) {
        skp = 0.0f;  // a slot that was never written: its scales are not data
        lsv = 0.0f;
        rsv = 0.0f;
      }
      s_ops[half][lane] = floatx4{skp, lsv, rsv, 0.0f};
    }
  };

  // ---- consumer side ----
  floatx4 S[NT][4];
  Operand pb[NT][2 * EB];  // unquantized: a probability goes in as two bf16 terms (hi, lo)
  auto load_op = [&](const half8& bits) {
    if constexpr (PLAIN) return __builtin_bit_cast(bf16x8, bits);
    else return bits;
  };
  auto mma = [&](const Operand& a, const Operand& b, const floatx4& c) {
    if constexpr (PLAIN) return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
  };
  auto qk = [&](int half) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int u = 0; u < 4; ++u) S[nt][u] = floatx4{0.f, 0.f, 0.f, 0.f};
    // step by step over the channels: eight independent instructions (4 quads x 2 row tiles)
    // per step, the next step's four operands read from LDS while they run.  The scheduling
    // barriers keep that order; left alone, the compiler reads two operands, waits, issues
    // four instructions and so exposes the LDS latency eight times per group.
    Operand a[2][4];
#pragma unroll
    for (int u = 0; u < 4; ++u) a[0][u] = load_op(k_ops[half][u][0][lane]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      if (s + 1 < KS) {
#pragma unroll
        for (int u = 0; u < 4; ++u) a[(s + 1) & 1][u] = load_op(k_ops[half][u][s + 1][lane]);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          S[nt][u] = mma(a[s & 1][u], qb[nt][s], S[nt][u]);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto softmax_impl = [&](auto TAILC, int g, int half) {
    constexpr bool TAIL = decltype(TAILC)::value;
    const int pos0 = g << 6;
    float skp = p.scale_log2, lsv = 0.0f, rsv = 1.0f;
    if constexpr (!PLAIN) {
      const floatx4 sc = s_ops[half][lane];
      skp = sc[0];
      lsv = sc[1];
      rsv = sc[2];
    }
    online_softmax<MODE, NT, DT, TAIL>(S, skp, lsv, rsv, pos0 + 16 * g4, nrow, m_run, l_run, acc, pb);
  };
  auto pv = [&](int half) {
    // two channel tiles at a time: their four operands are read while the previous pair's
    // eight instructions run; the instructions alternate between four accumulators
    Operand a[2][2][2];
#pragma unroll
    for (int x = 0; x < 2; ++x)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) a[0][x][hf] = load_op(v_ops[half][x][hf][lane]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t2 = 0; t2 < DT / 2; ++t2) {
      if (t2 + 1 < DT / 2) {
#pragma unroll
        for (int x = 0; x < 2; ++x)
#pragma unroll
          for (int hf = 0; hf < 2; ++hf)
            a[(t2 + 1) & 1][x][hf] = load_op(v_ops[half][2 * (t2 + 1) + x][hf][lane]);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int x = 0; x < 2; ++x)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            acc[nt][2 * t2 + x] = mma(a[t2 & 1][x][hf], pb[nt][hf], acc[nt][2 * t2 + x]);
            if constexpr (PLAIN)
              acc[nt][2 * t2 + x] = mma(a[t2 & 1][x][hf], pb[nt][2 + hf], acc[nt][2 * t2 + x]);
          }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // ---- the walk: group g is consumed from half g % 2 while group g + 1 is converted into the
  // other half and group g + 2 is requested (indices past the end repeat the last group) ----
  Entries e_next, e_after;
  {
    Entries e0;
    fetch_entries(g0, e0);
    fetch_entries(min(g0 + 1, ng - 1), e_next);
    issue_loads(g0, e0);
  }
  publish(g0, 0);
  issue_loads(min(g0 + 1, ng - 1), e_next);
  fetch_entries(min(g0 + 2, ng - 1), e_after);
  __syncthreads();
  for (int g = g0; g < ng; ++g) {
    const int half = (g - g0) & 1;
    if (wave_live) {
      qk(half);
      if ((g << 6) + 64 > n_min) softmax_impl(std::true_type{}, g, half);
      else softmax_impl(std::false_type{}, g, half);
      pv(half);
    }
    // group g + 1 (requested one iteration ago) into the other half; request group g + 2
    publish(min(g + 1, ng - 1), half ^ 1);
    issue_loads(min(g + 2, ng - 1), e_after);
    fetch_entries(min(g + 3, ng - 1), e_after);
    __syncthreads();
  }

  if constexpr (PREFIX) {
    // ---- partials: slot = wavefronts + (1 + piece) * pairs + the row's pair, as the reduce
    // expects them ----
    const int rt = 16 * p.row_tiles;
    const size_t slot0 = (size_t)p.num_waves + (size_t)(chunk + 1) * p.batch * p.pairs_per_seq;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const float l = xor16_sum(l_run[nt]);
      const int rs = r0 + nt * 16 + m16;
      if (rs >= all_rows) continue;
      const int br = rs / p.rows, r = rs - br * p.rows;
      const int rg = r / rt, rl = r - rg * rt;
      const size_t row =
          (slot0 + (size_t)br * p.pairs_per_seq + h * p.num_row_groups + rg) * rt + rl;
      float* arow = p.ws_acc + row * D;
#pragma unroll
      for (int tt = 0; tt < DT; ++tt) *(floatx4*)(arow + 16 * tt + 4 * g4) = acc[nt][tt];
      if (g4 == 0) {
        p.ws_ml[row * 2] = m_run[nt];
        p.ws_ml[row * 2 + 1] = l;
      }
    }
    return;
  }
  // ---- normalised rows ----
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const float l = xor16_sum(l_run[nt]);
    const int r = r0 + nt * 16 + m16;
    if (r >= p.rows) continue;
    const int j = r / G, gi = r - j * G;
    float* orow = p.out + (((size_t)b * p.q_len + j) * p.num_q_heads + (size_t)h * G + gi) * D;
    const float inv = 1.0f / l;
#pragma unroll
    for (int tt = 0; tt < DT; ++tt) *(floatx4*)(orow + 16 * tt + 4 * g4) = acc[nt][tt] * inv;
  }
}

}  // namespace

bool prefill_applies(const AttnArgs& a) {
  // (the group-scaled int4 format has no many-row kernel: its row groups go through the
  // streaming kernel)
  return a.rows >= kRowsPerWorkgroup && a.mode != KVQ_INT4_GROUP32;
}

template <bool PREFIX>
hipError_t launch_many_rows(const AttnArgs& a, int all_rows, int walks, hipStream_t stream) {
  const int row_blocks = (all_rows + kRowsPerWorkgroup - 1) / kRowsPerWorkgroup;
  const dim3 grid((unsigned)((size_t)walks * a.num_kv_heads * row_blocks));
  const dim3 block(64 * kWavesPerGroup);
#define KVQ_LAUNCH_PREFILL(MODE)                                                                \
  if (a.head_dim == 128)                                                                        \
    hipLaunchKernelGGL((attn_prefill_kernel<MODE, 128, PREFIX>), grid, block, 0, stream, a);    \
  else                                                                                          \
    hipLaunchKernelGGL((attn_prefill_kernel<MODE, 64, PREFIX>), grid, block, 0, stream, a)
  if (a.mode == KVQ_INT8_TOKEN_HEAD) {
    KVQ_LAUNCH_PREFILL(KVQ_INT8_TOKEN_HEAD);
  } else if (a.mode == KVQ_FP8E4M3_BLOCK_HEAD) {
    KVQ_LAUNCH_PREFILL(KVQ_FP8E4M3_BLOCK_HEAD);
  } else if (a.mode == KVQ_BF16_PLAIN) {
    KVQ_LAUNCH_PREFILL(KVQ_BF16_PLAIN);
  } else if (a.mode == KVQ_INT4_TOKEN_HEAD) {  // (head_dim 128 only)
    hipLaunchKernelGGL((attn_prefill_kernel<KVQ_INT4_TOKEN_HEAD, 128, PREFIX>), grid, block, 0,
                       stream, a);
  } else {
    KVQ_LAUNCH_PREFILL(KVQ_FP8E4M3_TENSOR);
  }
#undef KVQ_LAUNCH_PREFILL
  return hipGetLastError();
}

hipError_t launch_prefill(const AttnArgs& a, hipStream_t stream) {
  return launch_many_rows<false>(a, a.rows, a.batch, stream);
}

// the shared groups of a decode or verification batch (a.shared_groups > 0), ahead of the
// streaming kernel
hipError_t launch_prefix(const AttnArgs& a, hipStream_t stream) {
  return launch_many_rows<true>(a, a.batch * a.rows, a.prefix_chunks, stream);
}

}  // namespace kvq
