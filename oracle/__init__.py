"""CPU oracle for the quantized KV-cache write and quantized paged decode attention.

TEST INFRASTRUCTURE.  Only tests, the smoke check and the benchmark's CPU-baseline
leg import this package.  It is a thin numpy/ctypes front for `kvq_oracle.c` (plain
C, fp64) and shares nothing with the GPU library.

Arrays use the oracle's canonical layout:
  cache  uint8   [num_blocks, 2, num_kv_heads, block_size, head_dim]   (0 = K, 1 = V)
  scales float32 [num_blocks, 2, num_kv_heads, block_size]   mode 0 (int8 per token-head)
         float32 [num_blocks, 2, num_kv_heads]               mode 1 (fp8-e4m3 per block-head)
  k, v, q uint16 bf16 bit patterns [tokens, heads, head_dim]
Mode 2 is the unquantized baseline: cache uint16 (bf16 bit patterns), same shape; scales is an
empty float32 array.  Mode 3 is fp8-e4m3 with static per-tensor scales: scales is float32 [2]
(K, V), set by the caller and only read.  Mode 4 is int4 per token-head: cache rows are
head_dim / 2 bytes (channel 2j in the low nibble of byte j, channel 2j+1 in the high one,
4-bit two's complement), scales as mode 0.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

MODE_INT8 = 0
MODE_FP8 = 1
MODE_BF16 = 2
MODE_FP8_TENSOR = 3
MODE_INT4 = 4
MODE_INT4_GROUP = 5   # int4 codes, one scale per (token, kv head, 32 adjacent channels)
INT4_MODES = (MODE_INT4, MODE_INT4_GROUP)

_lib = None


def lib():
    global _lib
    if _lib is None:
        # KVQ_ORACLE_SO: load this build instead (tests/test_oracle_mutants.py runs the pins
        # against deliberately wrong copies of the source to show that they notice)
        _lib = _load(os.environ.get("KVQ_ORACLE_SO") or _build.build())
    return _lib


class use_library:
    """Context manager for tests of the tests: inside it every function of this package runs
    on the given build of the C source (a copy with a planted mistake) instead of the real one."""

    def __init__(self, so_path):
        self.mutant = _load(so_path)

    def __enter__(self):
        global _lib
        self.saved, _lib = lib(), self.mutant
        return self

    def __exit__(self, *exc):
        global _lib
        _lib = self.saved
        return False


def _load(path):
    L = C.CDLL(path)
    L.oracle_bf16_to_f64.restype = C.c_double
    L.oracle_bf16_to_f64.argtypes = [C.c_uint16]
    L.oracle_fp8_decode.restype = C.c_double
    L.oracle_fp8_decode.argtypes = [C.c_uint8]
    L.oracle_fp8_encode.restype = C.c_uint8
    L.oracle_fp8_encode.argtypes = [C.c_double]
    L.oracle_int8_encode.restype = C.c_int8
    L.oracle_int8_encode.argtypes = [C.c_double, C.c_float]
    L.oracle_int4_encode.restype = C.c_int8
    L.oracle_int4_encode.argtypes = [C.c_double, C.c_float]
    L.oracle_scale.restype = C.c_float
    L.oracle_scale.argtypes = [C.c_double, C.c_double]
    L.oracle_kv_quant_write.restype = C.c_int
    L.oracle_kv_quant_write.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                        C.c_void_p, C.c_void_p] + [C.c_int32] * 5
    L.oracle_dequant_at.restype = C.c_double
    L.oracle_dequant_at.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int,
                                    C.c_int, C.c_int, C.c_int, C.c_int32, C.c_int32, C.c_int32]
    L.oracle_gather_dequant.restype = None
    L.oracle_gather_dequant.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                                        C.c_int32, C.c_int, C.c_int, C.c_int32, C.c_int32,
                                        C.c_int32, C.c_void_p]
    L.oracle_paged_decode_attn.restype = C.c_int
    L.oracle_paged_decode_attn.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p] + \
        [C.c_int32] * 5 + [C.c_void_p, C.c_int32, C.c_void_p] + [C.c_int32] * 3 + \
        [C.c_double, C.c_void_p]
    L.oracle_attn_weights.restype = C.c_int32
    L.oracle_attn_weights.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p] + [C.c_int32] * 4 + \
        [C.c_void_p] + [C.c_int32] * 6 + [C.c_double, C.c_void_p]
    L.oracle_num_threads.restype = C.c_int
    L.oracle_num_threads.argtypes = []
    return L


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def _chk(a, dtype, name):
    if not isinstance(a, np.ndarray) or a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError("%s must be a C-contiguous numpy array of %s" % (name, np.dtype(dtype)))
    return a


def bf16_to_f64(bits):
    """Exact widening of bf16 bit patterns (uint16) to float64."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def fp8_decode(codes):
    codes = np.asarray(codes, dtype=np.uint8)
    L = lib()
    out = np.empty(codes.shape, dtype=np.float64)
    flat, o = codes.reshape(-1), out.reshape(-1)
    for i in range(flat.size):
        o[i] = L.oracle_fp8_decode(int(flat[i]))
    return out


def fp8_encode(y):
    y = np.asarray(y, dtype=np.float64)
    L = lib()
    out = np.empty(y.shape, dtype=np.uint8)
    flat, o = y.reshape(-1), out.reshape(-1)
    for i in range(flat.size):
        o[i] = L.oracle_fp8_encode(float(flat[i]))
    return out


def int8_encode(x, s):
    """RNE(x / s) clamped to [-127, 127]; x float64 array, s one fp32 scale."""
    x = np.asarray(x, dtype=np.float64)
    L = lib()
    out = np.empty(x.shape, dtype=np.int8)
    flat, o = x.reshape(-1), out.reshape(-1)
    for i in range(flat.size):
        o[i] = L.oracle_int8_encode(float(flat[i]), float(np.float32(s)))
    return out


def int4_encode(x, s):
    """RNE(x / s) clamped to [-7, 7]; x float64 array, s one fp32 scale."""
    x = np.asarray(x, dtype=np.float64)
    L = lib()
    out = np.empty(x.shape, dtype=np.int8)
    flat, o = x.reshape(-1), out.reshape(-1)
    for i in range(flat.size):
        o[i] = L.oracle_int4_encode(float(flat[i]), float(np.float32(s)))
    return out


def unpack_int4(cache):
    """int8 codes [..., 2 * n] of an int4 cache [..., n] (low nibble first)."""
    lo = (cache & 15).astype(np.int8)
    hi = (cache >> 4).astype(np.int8)
    both = np.stack([lo, hi], axis=-1).reshape(cache.shape[:-1] + (2 * cache.shape[-1],))
    return ((both ^ 8) - 8).astype(np.int8)


def head_dim_of(cache, mode):
    return cache.shape[-1] * (2 if mode in INT4_MODES else 1)


def scale(absmax, qmax):
    return np.float32(lib().oracle_scale(float(absmax), float(qmax)))


def alloc_cache(mode, num_blocks, block_size, num_kv_heads, head_dim):
    """Zero-filled canonical cache and scales."""
    cache = np.zeros((num_blocks, 2, num_kv_heads, block_size,
                      head_dim // 2 if mode in INT4_MODES else head_dim),
                     dtype=np.uint16 if mode == MODE_BF16 else np.uint8)
    if mode == MODE_BF16:
        scales = np.zeros((0,), dtype=np.float32)
    elif mode == MODE_FP8_TENSOR:
        scales = np.zeros((2,), dtype=np.float32)
    elif mode in (MODE_INT8, MODE_INT4):
        scales = np.zeros((num_blocks, 2, num_kv_heads, block_size), dtype=np.float32)
    elif mode == MODE_INT4_GROUP:
        scales = np.zeros((num_blocks, 2, num_kv_heads, block_size, head_dim // 32), dtype=np.float32)
    else:
        scales = np.zeros((num_blocks, 2, num_kv_heads), dtype=np.float32)
    return cache, scales


def _chk_cache(cache, scales, mode):
    _chk(cache, np.uint16 if mode == MODE_BF16 else np.uint8, "cache")
    _chk(scales, np.float32, "scales")
    nblk, two, H, bs, D = cache.shape
    assert two == 2
    assert scales.shape == {MODE_INT8: (nblk, 2, H, bs), MODE_FP8: (nblk, 2, H),
                            MODE_BF16: (0,), MODE_FP8_TENSOR: (2,),
                            MODE_INT4: (nblk, 2, H, bs),
                            MODE_INT4_GROUP: (nblk, 2, H, bs, D // 16)}[mode]


def kv_quant_write(k, v, slot_mapping, cache, scales, mode):
    """In-place write of bf16 rows k, v [T, H_kv, D] at slot_mapping [T] (int64)."""
    _chk(k, np.uint16, "k"), _chk(v, np.uint16, "v")
    _chk(slot_mapping, np.int64, "slot_mapping")
    _chk_cache(cache, scales, mode)
    nblk, two, H, bs, _ = cache.shape
    D = head_dim_of(cache, mode)
    assert k.shape == v.shape == (slot_mapping.shape[0], H, D)
    live = slot_mapping[slot_mapping >= 0]
    assert live.size == 0 or int(live.max()) < nblk * bs
    rc = lib().oracle_kv_quant_write(_ptr(k), _ptr(v), _ptr(slot_mapping), k.shape[0],
                                     _ptr(cache), _ptr(scales), mode, nblk, bs, H, D)
    if rc != 0:
        raise ValueError("oracle_kv_quant_write failed: %d" % rc)


def dequant(cache, scales, mode):
    """Dequantized fp64 value of every logical element, same shape as cache."""
    nblk, _, H, bs, D = cache.shape
    if mode == MODE_BF16:
        return bf16_to_f64(cache)
    if mode == MODE_INT4:
        return unpack_int4(cache).astype(np.float64) * scales.astype(np.float64)[..., None]
    if mode == MODE_INT4_GROUP:
        return unpack_int4(cache).astype(np.float64) * np.repeat(scales.astype(np.float64), 32, axis=-1)
    if mode == MODE_INT8:
        return cache.view(np.int8).astype(np.float64) * scales.astype(np.float64)[..., None]
    table = fp8_decode(np.arange(256, dtype=np.uint8))
    if mode == MODE_FP8_TENSOR:
        return table[cache] * scales.astype(np.float64)[None, :, None, None, None]
    return table[cache] * scales.astype(np.float64)[..., None, None]


def gather_dequant(cache, scales, mode, block_table_row, n, kv, h):
    """Dense fp64 [n, D] of K (kv=0) or V (kv=1) of one sequence and kv head."""
    _chk_cache(cache, scales, mode)
    row = np.ascontiguousarray(block_table_row, dtype=np.int32)
    nblk, _, H, bs, _ = cache.shape
    D = head_dim_of(cache, mode)
    assert (n + bs - 1) // bs <= row.shape[0]
    assert n == 0 or (row[:(n + bs - 1) // bs].min() >= 0 and row[:(n + bs - 1) // bs].max() < nblk)
    dense = np.empty((n, D), dtype=np.float64)
    lib().oracle_gather_dequant(_ptr(cache), _ptr(scales), mode, _ptr(row), n, kv, h, bs, H, D,
                                _ptr(dense))
    return dense


def paged_decode_attn(q, cache, scales, mode, block_tables, seq_lens, q_len, sm_scale):
    """out float64 [batch*q_len, H_q, D]."""
    _chk(q, np.uint16, "q"), _chk_cache(cache, scales, mode)
    _chk(block_tables, np.int32, "block_tables"), _chk(seq_lens, np.int32, "seq_lens")
    nblk, _, H, bs, _ = cache.shape
    D = head_dim_of(cache, mode)
    batch = seq_lens.shape[0]
    assert q.shape[0] == batch * q_len and q.shape[2] == D
    Hq = q.shape[1]
    assert Hq % H == 0 and block_tables.shape[0] == batch
    for b in range(batch):
        nb = (int(seq_lens[b]) + bs - 1) // bs
        assert nb <= block_tables.shape[1]
        assert block_tables[b, :nb].min() >= 0 and block_tables[b, :nb].max() < nblk
    out = np.empty((batch * q_len, Hq, D), dtype=np.float64)
    rc = lib().oracle_paged_decode_attn(_ptr(q), _ptr(cache), _ptr(scales), mode, nblk, bs, H, D,
                                        _ptr(block_tables), block_tables.shape[1], _ptr(seq_lens),
                                        batch, q_len, Hq, float(sm_scale), _ptr(out))
    if rc != 0:
        raise ValueError("oracle_paged_decode_attn failed: %d" % rc)
    return out


def attn_weights(q, cache, scales, mode, block_table_row, seq_len, q_len, j, hq, q_token_index,
                 sm_scale):
    """Softmax weights of one (sequence, query token j, q head hq): float64 [n]."""
    _chk(q, np.uint16, "q"), _chk_cache(cache, scales, mode)
    row = np.ascontiguousarray(block_table_row, dtype=np.int32)
    nblk, _, H, bs, _ = cache.shape
    D = head_dim_of(cache, mode)
    n = seq_len - q_len + j + 1
    w = np.empty(n, dtype=np.float64)
    got = lib().oracle_attn_weights(_ptr(q), _ptr(cache), _ptr(scales), mode, bs, H, D, _ptr(row),
                                    seq_len, q_len, j, q.shape[1], hq, q_token_index,
                                    float(sm_scale), _ptr(w))
    assert got == n
    return w


def blocks_export(cache, scales, mode, block_ids):
    """Packed copy of the named blocks (the tiered cache's eviction to CPU memory, Section 3.3):
    packed block i is pool block block_ids[i].  Returns (packed cache, packed scales)."""
    _chk_cache(cache, scales, mode)
    ids = np.asarray(block_ids, dtype=np.int64)
    assert ids.size == 0 or (ids.min() >= 0 and ids.max() < cache.shape[0])
    per_block = mode in (MODE_INT8, MODE_FP8, MODE_INT4, MODE_INT4_GROUP)  # else the scales are not part of a block
    packed_scales = scales[ids].copy() if per_block else scales.copy()
    return cache[ids].copy(), packed_scales


def blocks_import(packed_cache, packed_scales, mode, block_ids, cache, scales):
    """The reverse (LoadToGPU of Algorithm 1): pool block block_ids[i] becomes packed block i,
    in place; every other block keeps its contents.  The ids must differ."""
    _chk_cache(cache, scales, mode)
    ids = np.asarray(block_ids, dtype=np.int64)
    assert len(set(ids.tolist())) == ids.size
    assert ids.size == 0 or (ids.min() >= 0 and ids.max() < cache.shape[0])
    for i, blk in enumerate(ids):
        cache[blk] = packed_cache[i]
        if mode in (MODE_INT8, MODE_FP8, MODE_INT4, MODE_INT4_GROUP):
            scales[blk] = packed_scales[i]


def num_threads():
    return int(lib().oracle_num_threads())
