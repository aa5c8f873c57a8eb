"""Seeded synthetic workloads shaped like the benchmark configurations.

This module only draws inputs (shapes, lengths, block tables, bf16 bit patterns) and
counts bytes.  It holds none of the method's arithmetic (no quantization, no attention)
and is the one module both the GPU tests/bench and the CPU checker's tests take their
inputs from, so that both sides see identical data.

All draws use numpy's PCG64 (`numpy.random.default_rng`) and are reproducible anywhere.
K/V rows are generated per sequence on demand, so the full-size configurations never
need all of K/V in host memory at once.
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

MODE_INT8 = 0  # int8 codes, one fp32 scale per (token, kv head)
MODE_FP8 = 1   # fp8-e4m3 codes, one fp32 scale per (block, kv head)
MODE_BF16 = 2  # the unquantized baseline: bf16 rows stored as they are, no scales
MODE_FP8_TENSOR = 3  # fp8-e4m3 codes, static scales: one for a layer's K, one for its V
MODE_INT4 = 4  # int4 codes in [-7, 7], two per byte, one fp32 scale per (token, kv head)
MODE_INT4_GROUP = 5  # int4 codes, one fp32 scale per (token, kv head, 32 adjacent channels)

# Static scales for the generators' data: |K| reaches about 20 * 4.6 in the outlier channels and
# |V| about 6 (N(0,1) over ~1e9 draws), against the format's 448; a few V values saturate.
STATIC_SCALES = (0.25, 0.0125)

BASE_SEED = 26052963900


def to_bf16_bits(x):
    """Round float32 values to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Workload:
    name: str
    mode: int
    batch: int
    q_len: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    block_size: int
    seq_lens: np.ndarray            # int32 [batch], counts the q_len current tokens
    block_tables: np.ndarray        # int32 [batch, max_blocks], -1 where unused
    num_blocks: int                 # physical blocks in the pool
    seed: int
    outlier_channels: np.ndarray    # flat indices into [num_kv_heads * head_dim] of K channels x20
    shared_prefix: int = 0          # leading positions whose blocks every sequence shares
    append_tokens: int = 0          # tokens per sequence written by a separate append call
    chunk_tokens: int = 0           # split-K chunk the configuration names (0 = library default)
    q: Optional[np.ndarray] = field(default=None, repr=False)  # uint16 [batch*q_len, H_q, D]

    @property
    def sm_scale(self):
        return 1.0 / float(np.sqrt(self.head_dim))

    @property
    def max_seq_len(self):
        return int(self.seq_lens.max()) if self.batch else 0

    @property
    def group(self):
        return self.num_q_heads // self.num_kv_heads

    def slots(self, b, start, stop):
        """Physical slots (int64) of positions start..stop-1 of sequence b."""
        p = np.arange(start, stop, dtype=np.int64)
        return self.block_tables[b, p // self.block_size].astype(np.int64) * self.block_size \
            + p % self.block_size

    def kv_rows(self, b, start, stop):
        """bf16 bit patterns (k, v), each uint16 [stop-start, H_kv, D], of positions
        start..stop-1 of sequence b.  Positions inside the shared prefix are the same for
        every sequence.  Deterministic in (seed, b, position)."""
        H, D = self.num_kv_heads, self.head_dim
        k = np.empty((stop - start, H, D), dtype=np.uint16)
        v = np.empty((stop - start, H, D), dtype=np.uint16)
        gain = np.ones(H * D, dtype=np.float32)
        gain[self.outlier_channels] = 20.0
        gain = gain.reshape(1, H, D)
        # generated in fixed pieces of 256 positions so any [start, stop) gives the same values
        piece = 256
        for p0 in range((start // piece) * piece, stop, piece):
            owner = -1 if p0 + piece <= self.shared_prefix else b
            rng = np.random.default_rng([self.seed, owner + 1, p0 // piece])
            kk = rng.standard_normal((piece, H, D), dtype=np.float32) * gain
            vv = rng.standard_normal((piece, H, D), dtype=np.float32)
            lo, hi = max(p0, start), min(p0 + piece, stop)
            k[lo - start:hi - start] = to_bf16_bits(kk[lo - p0:hi - p0])
            v[lo - start:hi - start] = to_bf16_bits(vv[lo - p0:hi - p0])
        return k, v

    def prefill_len(self, b):
        """Positions of sequence b written before the append call."""
        return int(self.seq_lens[b]) - self.append_tokens

    def write_range(self, b):
        """(start, stop) of the positions sequence b itself has to write during prefill:
        sequence 0 also writes the shared prefix, the others start after it."""
        start = 0 if b == 0 else self.shared_prefix
        return start, self.prefill_len(b)

    def unique_tokens(self):
        """Stored positions counted once (a shared prefix counts once)."""
        total = int(self.seq_lens.astype(np.int64).sum())
        return total - (self.batch - 1) * self.shared_prefix if self.batch else 0

    def algorithmic_bytes(self):
        """Bytes one attention call has to move: codes and scales of every stored position
        once, q, out, the block-table entries used and seq_lens."""
        H, D, bs = self.num_kv_heads, self.head_dim, self.block_size
        if self.mode == MODE_INT8:
            per_token_head = 2.0 * (D + 4)
        elif self.mode == MODE_BF16:
            per_token_head = 4.0 * D
        elif self.mode == MODE_FP8_TENSOR:
            per_token_head = 2.0 * D
        elif self.mode == MODE_INT4:
            per_token_head = 2.0 * (D / 2 + 4)
        elif self.mode == MODE_INT4_GROUP:
            per_token_head = 2.0 * (D / 2 + 4 * (D / 32))
        else:
            per_token_head = 2.0 * D + 8.0 / bs
        kv = self.unique_tokens() * H * per_token_head
        rows = self.batch * self.q_len * self.num_q_heads * D
        tables = int(((self.seq_lens.astype(np.int64) + bs - 1) // bs).sum()) * 4
        total = kv + rows * 6.0 + tables + 4.0 * self.batch
        # "logical": a shared prefix counted once per sequence that reads it
        logical_kv = int(self.seq_lens.astype(np.int64).sum()) * H * per_token_head
        return {"kv": kv, "q_out": rows * 6.0, "tables": tables + 4.0 * self.batch,
                "total": total, "logical_total": total - kv + logical_kv}


def _tables(rng, seq_lens, block_size, shared_prefix=0, pool_factor=2):
    """Random permuted block tables over a pool of pool_factor x the needed blocks."""
    nb = (seq_lens.astype(np.int64) + block_size - 1) // block_size
    shared_blocks = shared_prefix // block_size
    own = nb - shared_blocks if shared_blocks else nb
    needed = int(own.sum()) + shared_blocks
    pool = max(pool_factor * needed, 1)
    perm = rng.permutation(pool).astype(np.int32)
    max_blocks = int(nb.max()) if len(nb) else 0
    tables = np.full((len(seq_lens), max_blocks), -1, dtype=np.int32)
    cursor = 0
    shared = perm[:shared_blocks]
    cursor += shared_blocks
    for b in range(len(seq_lens)):
        tables[b, :shared_blocks] = shared
        n_own = int(own[b])
        tables[b, shared_blocks:shared_blocks + n_own] = perm[cursor:cursor + n_own]
        cursor += n_own
    return tables, pool


def _finish(name, mode, rng, seed, seq_lens, q_len, Hq, Hkv, D, bs, outliers=True,
            shared_prefix=0, append_tokens=0, chunk_tokens=0, num_blocks=None, tables=None):
    seq_lens = np.asarray(seq_lens, dtype=np.int32)
    assert shared_prefix % 256 == 0 and shared_prefix % bs == 0
    assert shared_prefix == 0 or int(seq_lens.min()) - append_tokens >= shared_prefix
    if tables is None:
        tables, pool = _tables(rng, seq_lens, bs, shared_prefix)
    else:
        pool = num_blocks
    n_out = max(1, (Hkv * D) // 100) if outliers else 0
    out_ch = np.sort(rng.choice(Hkv * D, size=n_out, replace=False)) if n_out else \
        np.zeros(0, dtype=np.int64)
    q = to_bf16_bits(rng.standard_normal((len(seq_lens) * q_len, Hq, D), dtype=np.float32))
    return Workload(name=name, mode=mode, batch=len(seq_lens), q_len=q_len, num_q_heads=Hq,
                    num_kv_heads=Hkv, head_dim=D, block_size=bs, seq_lens=seq_lens,
                    block_tables=tables, num_blocks=pool, seed=seed, outlier_channels=out_ch,
                    shared_prefix=shared_prefix, append_tokens=append_tokens,
                    chunk_tokens=chunk_tokens, q=q)


def tiny(mode=MODE_INT8):
    """Batch 2, seq_lens {37, 100}, 4 q heads, 2 kv heads, D 64, bs 16, pool of 16 blocks."""
    seed = BASE_SEED + 1
    rng = np.random.default_rng(seed)
    seq_lens = np.array([37, 100], dtype=np.int32)
    perm = rng.permutation(16).astype(np.int32)
    tables = np.full((2, 7), -1, dtype=np.int32)
    tables[0, :3] = perm[:3]
    tables[1, :7] = perm[3:10]
    return _finish("tiny", mode, rng, seed, seq_lens, 1, 4, 2, 64, 16, outliers=False,
                   num_blocks=16, tables=tables)


def llama8b(batch=64, lo=512, hi=4096, mode=MODE_INT8, seed_offset=0):
    """32 q heads, 8 kv heads, D 128, bs 16; seq_lens uniform in [lo, hi]; int8 per token-head."""
    seed = BASE_SEED + 2 + 1000 * seed_offset
    rng = np.random.default_rng(seed)
    seq_lens = rng.integers(lo, hi + 1, size=batch)
    return _finish("llama3_8b_layer", mode, rng, seed, seq_lens, 1, 32, 8, 128, 16)


def fp8_append(batch=256, lo=1024, hi=8192, mode=MODE_FP8):
    """Same heads, fp8-e4m3 per block-head; cache holds L tokens, then one token per sequence
    is appended; seq_lens here already count the appended token."""
    seed = BASE_SEED + 3
    rng = np.random.default_rng(seed)
    seq_lens = rng.integers(lo, hi + 1, size=batch) + 1
    return _finish("fp8_append", mode, rng, seed, seq_lens, 1, 32, 8, 128, 16,
                   append_tokens=1)


def long_gqa(batch=32, lo=16384, hi=65536, mode=MODE_INT8):
    """64 q heads, 4 kv heads, D 128, bs 64; seq_lens log-uniform in [lo, hi]; split-K 2048."""
    seed = BASE_SEED + 4
    rng = np.random.default_rng(seed)
    seq_lens = np.floor(np.exp(rng.uniform(np.log(lo), np.log(hi), size=batch))).astype(np.int64)
    return _finish("long_gqa", mode, rng, seed, seq_lens, 1, 64, 4, 128, 64, chunk_tokens=2048)


def verify_prefix(batch=128, lo=2048, hi=16384, mode=MODE_INT8, shared_prefix=1024):
    """64 q heads, 8 kv heads, D 128, bs 16, 4 causal query tokens; the first shared_prefix
    positions' blocks are shared by all sequences.  mode selects the layer parity
    (even layers int8 per token-head, odd layers fp8 per block-head)."""
    seed = BASE_SEED + 5
    rng = np.random.default_rng(seed)
    seq_lens = rng.integers(lo, hi + 1, size=batch)
    return _finish("verify_prefix", mode, rng, seed, seq_lens, 4, 64, 8, 128, 16,
                   shared_prefix=shared_prefix)


def chunk_prefill(mode=MODE_INT8, batch=8, chunk=512, prefix=4096, Hq=32, Hkv=8, D=128, bs=16):
    """A chunk of a prompt per sequence: `chunk` query tokens attending causally over a
    `prefix`-token context already in the cache and over themselves (Section 2's prefill phase
    cut into chunks, fed from the Section 7.2.2 cache); configuration 2's heads by default."""
    return custom("chunk_prefill", mode, [prefix + chunk] * batch, chunk, Hq, Hkv, D, bs, seed=5)


def custom(name, mode, seq_lens, q_len, Hq, Hkv, D, bs, seed, outliers=True, shared_prefix=0,
           append_tokens=0, chunk_tokens=0):
    """Any other shape, for parity cases (ragged tails, odd lengths, other group sizes)."""
    rng = np.random.default_rng(seed)
    return _finish(name, mode, rng, seed, seq_lens, q_len, Hq, Hkv, D, bs, outliers=outliers,
                   shared_prefix=shared_prefix, append_tokens=append_tokens,
                   chunk_tokens=chunk_tokens)
