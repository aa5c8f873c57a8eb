"""Python binding of the C-ABI library (include/kvq.h): argument marshalling only.

Every step of the path runs in the library's HIP kernels; torch tensors are used for
device memory and for the current stream.  There is no CPU fallback: if the built library
is missing, loading fails with an error.
"""
import ctypes as C
import os

MODE_INT8 = 0   # KVQ_INT8_TOKEN_HEAD
MODE_FP8 = 1    # KVQ_FP8E4M3_BLOCK_HEAD
MODE_BF16 = 2   # KVQ_BF16_PLAIN (unquantized baseline)
MODE_FP8_TENSOR = 3  # KVQ_FP8E4M3_TENSOR (static per-tensor scales)
MODE_INT4 = 4    # KVQ_INT4_TOKEN_HEAD (head_dim 128)
MODE_INT4_GROUP = 5   # KVQ_INT4_GROUP32 (head_dim 128; one scale per 32 channels)

OK, E_NULLPTR, E_BAD_MODE, E_BAD_SHAPE, E_WORKSPACE, E_HIP, E_BAD_INDEX = 0, -1, -2, -3, -4, -5, -6

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libkvq.so")

EXPORTS = ("kvq_cache_bytes", "kvq_scales_bytes", "kv_quant_write",
           "paged_decode_attn_workspace_bytes", "paged_decode_attn_prefix_workspace_bytes",
           "paged_decode_attn", "paged_decode_attn_prefix", "paged_decode_attn_static",
           "kvq_cache_to_canonical", "kvq_cache_from_canonical",
           "kvq_blocks_export", "kvq_blocks_import",
           "kvq_strerror")
# what the measurement build (libkvq_prof.so, include/kvq_prof.h) exports on top
PROF_EXPORTS = ("kvq_profile_split_events", "kvq_profile_read_ceiling", "kvq_profile_skip_reduce",
                "kvq_profile_prefill_kernel", "kvq_profile_wave_clock")
PROF_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libkvq_prof.so")


class CacheDesc(C.Structure):
    """kvq_cache_desc_t"""
    _fields_ = [("mode", C.c_int32), ("num_blocks", C.c_int32), ("block_size", C.c_int32),
                ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32)]

    def cache_shape(self):
        return (self.num_blocks, 2, self.num_kv_heads, self.block_size,
                self.head_dim // 2 if self.mode in (MODE_INT4, MODE_INT4_GROUP) else self.head_dim)

    def scales_shape(self):
        if self.mode in (MODE_INT8, MODE_INT4):
            return (self.num_blocks, 2, self.num_kv_heads, self.block_size)
        if self.mode == MODE_INT4_GROUP:
            return (self.num_blocks, 2, self.num_kv_heads, self.block_size, self.head_dim // 32)
        if self.mode == MODE_BF16:
            return (0,)
        if self.mode == MODE_FP8_TENSOR:
            return (2,)
        return (self.num_blocks, 2, self.num_kv_heads)


class KvqError(RuntimeError):
    def __init__(self, code, what):
        super().__init__("%s failed: %d (%s)" % (what, code, strerror(code)))
        self.code = code


_lib = None
_prof_lib = None


def _load(path, prof):
    if not os.path.exists(path):
        raise RuntimeError(
            "%s is not built: run `python -m paper_2605_29639_amd.build` "
            "(there is no CPU fallback)" % path)
    L = C.CDLL(path)
    P, I32, SZ = C.c_void_p, C.c_int32, C.c_size_t
    D = C.POINTER(CacheDesc)
    L.kvq_cache_bytes.restype, L.kvq_cache_bytes.argtypes = SZ, [D]
    L.kvq_scales_bytes.restype, L.kvq_scales_bytes.argtypes = SZ, [D]
    L.kv_quant_write.restype = C.c_int
    L.kv_quant_write.argtypes = [P, P, P, I32, P, P, D, P]
    L.paged_decode_attn_workspace_bytes.restype = SZ
    L.paged_decode_attn_workspace_bytes.argtypes = [D, I32, I32, I32, I32, I32]
    L.paged_decode_attn_prefix_workspace_bytes.restype = SZ
    L.paged_decode_attn_prefix_workspace_bytes.argtypes = [D, I32, I32, I32, I32, I32, I32]
    L.paged_decode_attn.restype = C.c_int
    L.paged_decode_attn.argtypes = [P, P, P, D, P, I32, P, I32, I32, I32, I32, C.c_float,
                                    I32, P, P, SZ, P]
    L.paged_decode_attn_prefix.restype = C.c_int
    L.paged_decode_attn_prefix.argtypes = [P, P, P, D, P, I32, P, I32, I32, I32, I32, C.c_float,
                                           I32, I32, P, P, SZ, P]
    L.paged_decode_attn_static.restype = C.c_int
    L.paged_decode_attn_static.argtypes = [P, P, P, D, P, I32, P, I32, I32, I32, I32, C.c_float,
                                           I32, P, P]
    L.kvq_cache_to_canonical.restype = C.c_int
    L.kvq_cache_to_canonical.argtypes = [P, P, D, P]
    L.kvq_cache_from_canonical.restype = C.c_int
    L.kvq_cache_from_canonical.argtypes = [P, P, D, P]
    L.kvq_blocks_export.restype = C.c_int
    L.kvq_blocks_export.argtypes = [P, P, D, P, I32, P, P, P]
    L.kvq_blocks_import.restype = C.c_int
    L.kvq_blocks_import.argtypes = [P, P, D, P, I32, P, P, P]
    L.kvq_strerror.restype, L.kvq_strerror.argtypes = C.c_char_p, [C.c_int]
    if prof:
        L.kvq_profile_split_events.restype = None
        L.kvq_profile_split_events.argtypes = [P, P]
        L.kvq_profile_skip_reduce.restype = None
        L.kvq_profile_skip_reduce.argtypes = [C.c_int]
        L.kvq_profile_prefill_kernel.restype = None
        L.kvq_profile_prefill_kernel.argtypes = [C.c_int]
        L.kvq_profile_wave_clock.restype = None
        L.kvq_profile_wave_clock.argtypes = [P]
        L.kvq_profile_read_ceiling.restype = None
        L.kvq_profile_read_ceiling.argtypes = [C.c_int]
    return L


def lib():
    """The loaded library (raw ctypes handle)."""
    global _lib
    if _lib is None:
        _lib = _load(LIB_PATH, False)
    return _lib


def prof_lib():
    """The measurement build of the library (benchmarks and tests only): every entry point of
    lib() plus the switches of include/kvq_prof.h.  Pass it as `L=` to the wrappers below."""
    global _prof_lib
    if _prof_lib is None:
        _prof_lib = _load(PROF_LIB_PATH, True)
    return _prof_lib


def strerror(code):
    return lib().kvq_strerror(int(code)).decode()


def _stream(stream):
    if stream is not None:
        return C.c_void_p(int(stream))
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, name):
    import torch
    if t is not None and t.numel() == 0 and t.dtype == dtype:
        return C.c_void_p(None)  # an empty tensor has no storage to point at
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError("%s must be a contiguous device tensor of %s" % (name, dtype))
    return C.c_void_p(t.data_ptr())


def make_desc(mode, num_blocks, block_size, num_kv_heads, head_dim):
    return CacheDesc(int(mode), int(num_blocks), int(block_size), int(num_kv_heads), int(head_dim))


def alloc_cache(desc, device="cuda", zero=True):
    """(cache uint8, scales float32) device tensors of the sizes the library reports.  With
    zero=True every logical code and scale is 0 (int8 codes are stored as code + 128, so the
    bytes of an all-zero int8 cache are 0x80)."""
    import torch
    nbytes, sbytes = lib().kvq_cache_bytes(desc), lib().kvq_scales_bytes(desc)
    make = torch.zeros if zero else torch.empty
    cache = make(nbytes, dtype=torch.uint8, device=device)
    if zero and desc.mode == MODE_INT8:
        cache.fill_(0x80)
    if zero and desc.mode in (MODE_INT4, MODE_INT4_GROUP):
        cache.fill_(0x88)  # nibbles are stored as code + 8
    scales = make(sbytes // 4, dtype=torch.float32, device=device).view(desc.scales_shape())
    return cache, scales


_pool_sizes = {}   # descriptor fields -> (cache bytes, scales bytes), as the library reports them


def _check_pool(cache, scales, desc):
    """The cache and scales tensors have the sizes the library reports for the descriptor: a
    smaller buffer would be overrun on the device, which checks nothing."""
    key = (desc.mode, desc.num_blocks, desc.block_size, desc.num_kv_heads, desc.head_dim)
    sizes = _pool_sizes.get(key)
    if sizes is None:
        sizes = _pool_sizes[key] = (lib().kvq_cache_bytes(desc), lib().kvq_scales_bytes(desc))
    nbytes, sbytes = sizes
    if cache is None or cache.numel() * cache.element_size() != nbytes:
        raise ValueError("cache must hold exactly kvq_cache_bytes(desc) = %d bytes" % nbytes)
    have = 0 if scales is None else scales.numel() * scales.element_size()
    if have != sbytes:
        raise ValueError("scales must hold exactly kvq_scales_bytes(desc) = %d bytes, not %d"
                         % (sbytes, have))


def kv_quant_write(k, v, slot_mapping, cache, scales, desc, stream=None, L=None):
    import torch
    rows = (k.shape[0], desc.num_kv_heads, desc.head_dim)
    if tuple(k.shape) != rows or tuple(v.shape) != rows:
        raise ValueError("k and v must be [num_tokens, %d, %d], not %s and %s"
                         % (rows[1], rows[2], tuple(k.shape), tuple(v.shape)))
    if tuple(slot_mapping.shape) != (k.shape[0],):
        raise ValueError("slot_mapping must be [num_tokens] = [%d]" % k.shape[0])
    _check_pool(cache, scales, desc)
    rc = (L or lib()).kv_quant_write(_dev(k, torch.bfloat16, "k"), _dev(v, torch.bfloat16, "v"),
                              _dev(slot_mapping, torch.int64, "slot_mapping"), k.shape[0],
                              _dev(cache, torch.uint8, "cache"),
                              _dev(scales, torch.float32, "scales"), C.byref(desc),
                              _stream(stream))
    if rc != OK:
        raise KvqError(rc, "kv_quant_write")


def _check_attn_shapes(q, cache, scales, desc, block_tables, seq_lens, q_len, out):
    """Shapes the device code relies on without checking; returns the batch size."""
    if seq_lens.dim() != 1:
        raise ValueError("seq_lens must be [batch]")
    batch = seq_lens.shape[0]
    if q.dim() != 3 or q.shape[0] != batch * q_len or q.shape[2] != desc.head_dim:
        raise ValueError("q must be [batch * q_len, num_q_heads, %d] = [%d, *, %d], not %s"
                         % (desc.head_dim, batch * q_len, desc.head_dim, tuple(q.shape)))
    if tuple(out.shape) != tuple(q.shape):
        raise ValueError("out must have q's shape %s, not %s" % (tuple(q.shape), tuple(out.shape)))
    if block_tables.dim() != 2 or block_tables.shape[0] != batch:
        raise ValueError("block_tables must be [batch, max_blocks_per_seq] with batch = %d" % batch)
    _check_pool(cache, scales, desc)
    return batch


def workspace_bytes(desc, batch, q_len, num_q_heads, max_seq_len, chunk_tokens=0,
                    shared_prefix_tokens=0):
    """Bytes paged_decode_attn needs, or paged_decode_attn_prefix with shared_prefix_tokens."""
    if shared_prefix_tokens:
        return int(lib().paged_decode_attn_prefix_workspace_bytes(
            C.byref(desc), batch, q_len, num_q_heads, max_seq_len, chunk_tokens,
            int(shared_prefix_tokens)))
    return int(lib().paged_decode_attn_workspace_bytes(C.byref(desc), batch, q_len, num_q_heads,
                                                       max_seq_len, chunk_tokens))


def alloc_workspace(desc, batch, q_len, num_q_heads, max_seq_len, chunk_tokens=0, device="cuda",
                    shared_prefix_tokens=0):
    import torch
    n = workspace_bytes(desc, batch, q_len, num_q_heads, max_seq_len, chunk_tokens,
                        shared_prefix_tokens)
    return torch.empty(max(n, 16), dtype=torch.uint8, device=device)


def paged_decode_attn(q, cache, scales, desc, block_tables, seq_lens, q_len, max_seq_len,
                      sm_scale, out, workspace, chunk_tokens=0, stream=None, L=None,
                      shared_prefix_tokens=0):
    """paged_decode_attn, or paged_decode_attn_prefix when shared_prefix_tokens is given."""
    import torch
    batch = _check_attn_shapes(q, cache, scales, desc, block_tables, seq_lens, q_len, out)
    need = workspace_bytes(desc, batch, q_len, q.shape[1], max_seq_len, chunk_tokens,
                           shared_prefix_tokens)
    if batch > 0 and workspace.numel() * workspace.element_size() < need:
        raise ValueError("workspace holds %d bytes, the call needs %d" % (workspace.numel(), need))
    if shared_prefix_tokens:
        rc = (L or lib()).paged_decode_attn_prefix(
            _dev(q, torch.bfloat16, "q"), _dev(cache, torch.uint8, "cache"),
            _dev(scales, torch.float32, "scales"), C.byref(desc),
            _dev(block_tables, torch.int32, "block_tables"), block_tables.shape[1],
            _dev(seq_lens, torch.int32, "seq_lens"), batch, q_len, q.shape[1], max_seq_len,
            float(sm_scale), chunk_tokens, int(shared_prefix_tokens),
            _dev(out, torch.float32, "out"), _dev(workspace, torch.uint8, "workspace"),
            workspace.numel(), _stream(stream))
        if rc != OK:
            raise KvqError(rc, "paged_decode_attn_prefix")
        return
    rc = (L or lib()).paged_decode_attn(
        _dev(q, torch.bfloat16, "q"), _dev(cache, torch.uint8, "cache"),
        _dev(scales, torch.float32, "scales"), C.byref(desc),
        _dev(block_tables, torch.int32, "block_tables"), block_tables.shape[1],
        _dev(seq_lens, torch.int32, "seq_lens"), batch, q_len, q.shape[1], max_seq_len,
        float(sm_scale), chunk_tokens, _dev(out, torch.float32, "out"),
        _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream))
    if rc != OK:
        raise KvqError(rc, "paged_decode_attn")


STATIC_WORKSPACE_BYTES = 64 << 20   # KVQ_STATIC_WORKSPACE_BYTES


def paged_decode_attn_static(q, cache, scales, desc, block_tables, seq_lens, q_len, max_seq_len,
                             sm_scale, out, chunk_tokens=0, stream=None):
    """paged_decode_attn on the library's own static scratch buffer (no workspace argument)."""
    import torch
    batch = _check_attn_shapes(q, cache, scales, desc, block_tables, seq_lens, q_len, out)
    rc = lib().paged_decode_attn_static(
        _dev(q, torch.bfloat16, "q"), _dev(cache, torch.uint8, "cache"),
        _dev(scales, torch.float32, "scales"), C.byref(desc),
        _dev(block_tables, torch.int32, "block_tables"), block_tables.shape[1],
        _dev(seq_lens, torch.int32, "seq_lens"), batch, q_len, q.shape[1], max_seq_len,
        float(sm_scale), chunk_tokens, _dev(out, torch.float32, "out"), _stream(stream))
    if rc != OK:
        raise KvqError(rc, "paged_decode_attn_static")


def _any(t, dtype, name):
    """Device tensor, or pinned host tensor the GPU can address."""
    import torch
    if t is not None and t.numel() == 0 and t.dtype == dtype:
        return C.c_void_p(None)
    if not isinstance(t, torch.Tensor) or t.dtype != dtype or not t.is_contiguous() or \
            not (t.is_cuda or t.is_pinned()):
        raise TypeError("%s must be a contiguous device or pinned host tensor of %s" % (name, dtype))
    return C.c_void_p(t.data_ptr())


def packed_sizes(desc, num):
    """(cache bytes, scale floats) of `num` packed blocks."""
    nb = max(desc.num_blocks, 1)
    per_block_scales = desc.mode in (MODE_INT8, MODE_FP8, MODE_INT4, MODE_INT4_GROUP)
    return (num * (lib().kvq_cache_bytes(desc) // nb),
            num * (lib().kvq_scales_bytes(desc) // nb // 4) if per_block_scales else 0)


def blocks_export(cache, scales, desc, block_ids, packed_cache, packed_scales, stream=None):
    import torch
    rc = lib().kvq_blocks_export(_dev(cache, torch.uint8, "cache"), _dev(scales, torch.float32, "scales"),
                                 C.byref(desc), _dev(block_ids, torch.int32, "block_ids"),
                                 block_ids.numel(), _any(packed_cache, torch.uint8, "packed_cache"),
                                 _any(packed_scales, torch.float32, "packed_scales"), _stream(stream))
    if rc != OK:
        raise KvqError(rc, "kvq_blocks_export")


def blocks_import(packed_cache, packed_scales, desc, block_ids, cache, scales, stream=None):
    import torch
    rc = lib().kvq_blocks_import(_any(packed_cache, torch.uint8, "packed_cache"),
                                 _any(packed_scales, torch.float32, "packed_scales"), C.byref(desc),
                                 _dev(block_ids, torch.int32, "block_ids"), block_ids.numel(),
                                 _dev(cache, torch.uint8, "cache"), _dev(scales, torch.float32, "scales"),
                                 _stream(stream))
    if rc != OK:
        raise KvqError(rc, "kvq_blocks_import")


def cache_to_canonical(cache, desc, stream=None):
    """Canonical [num_blocks, 2, H_kv, block_size, head_dim] copy of a physical cache: uint8
    codes, or int16 bf16 bit patterns for an unquantized cache."""
    import torch
    out = torch.empty_like(cache)
    rc = lib().kvq_cache_to_canonical(_dev(cache, torch.uint8, "cache"), C.c_void_p(out.data_ptr()),
                                      C.byref(desc), _stream(stream))
    if rc != OK:
        raise KvqError(rc, "kvq_cache_to_canonical")
    if desc.mode == MODE_BF16:
        out = out.view(torch.int16)
    return out.view(desc.cache_shape())


def cache_from_canonical(canonical, desc, stream=None):
    """Physical-layout cache (flat uint8) holding the given canonical array."""
    import torch
    canonical = canonical.contiguous().view(-1).view(torch.uint8)
    out = torch.empty_like(canonical)
    rc = lib().kvq_cache_from_canonical(_dev(canonical, torch.uint8, "canonical"),
                                        C.c_void_p(out.data_ptr()), C.byref(desc), _stream(stream))
    if rc != OK:
        raise KvqError(rc, "kvq_cache_from_canonical")
    return out
