"""Shared by the tests: build an oracle-written cache for a workload (CPU only)."""
import numpy as np

import oracle
from paper_2605_29639_amd import workloads as W


def oracle_fill(wl, sequences=None):
    """Zero pool, then the oracle writes every sequence's prefill rows (one call per
    sequence, all of its tokens at once) and, if the workload has an append step, one
    more call carrying the appended token of every sequence.  With `sequences`, only
    those sequences are written (the rest of the pool stays zero)."""
    cache, scales = oracle.alloc_cache(wl.mode, wl.num_blocks, wl.block_size, wl.num_kv_heads,
                                       wl.head_dim)
    if wl.mode == W.MODE_FP8_TENSOR:
        scales[:] = W.STATIC_SCALES
    seqs = range(wl.batch) if sequences is None else sequences
    for b in seqs:
        start, stop = wl.write_range(b)
        if stop > start:
            k, v = wl.kv_rows(b, start, stop)
            oracle.kv_quant_write(k, v, wl.slots(b, start, stop), cache, scales, wl.mode)
    if wl.append_tokens:
        ks, vs, ss = [], [], []
        for b in seqs:
            p0, p1 = wl.prefill_len(b), int(wl.seq_lens[b])
            k, v = wl.kv_rows(b, p0, p1)
            ks.append(k), vs.append(v), ss.append(wl.slots(b, p0, p1))
        oracle.kv_quant_write(np.concatenate(ks), np.concatenate(vs), np.concatenate(ss), cache,
                              scales, wl.mode)
    return cache, scales


# --------------------------------------------------------------------------- GPU side

from paper_2605_29639_amd.fill import attn_err, bits_to_bf16_tensor, gpu_desc, gpu_fill  # noqa: E402,F401


def gpu_attention(wl, cache, scales, desc, chunk_tokens=None, seq_lens=None, q=None, q_len=None,
                  L=None, shared_prefix_tokens=0):
    """Run the library's paged_decode_attn on a device cache; returns float32 numpy out."""
    import torch
    from paper_2605_29639_amd import kvq
    q_len = wl.q_len if q_len is None else q_len
    seq_lens = wl.seq_lens if seq_lens is None else seq_lens
    qbits = wl.q if q is None else q
    chunk = wl.chunk_tokens if chunk_tokens is None else chunk_tokens
    max_len = int(seq_lens.max())
    qd = bits_to_bf16_tensor(qbits)
    bt = torch.from_numpy(wl.block_tables).cuda()
    sl = torch.from_numpy(np.ascontiguousarray(seq_lens, dtype=np.int32)).cuda()
    out = torch.full((qbits.shape[0], qbits.shape[1], wl.head_dim), float("nan"),
                     dtype=torch.float32, device="cuda")
    ws = kvq.alloc_workspace(desc, len(seq_lens), q_len, qbits.shape[1], max_len, chunk,
                             shared_prefix_tokens=shared_prefix_tokens)
    ws.fill_(0xFF)  # NaN patterns: the kernels must not depend on workspace contents
    kvq.paged_decode_attn(qd, cache, scales, desc, bt, sl, q_len, max_len, wl.sm_scale, out, ws,
                          chunk_tokens=chunk, L=L, shared_prefix_tokens=shared_prefix_tokens)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def upload_oracle_cache(wl, cache_np, scales_np):
    """Oracle-written canonical cache -> device tensors in the library's physical layout."""
    import torch
    from paper_2605_29639_amd import kvq
    desc = gpu_desc(wl)
    if cache_np.dtype == np.uint16:  # unquantized cache: bf16 bit patterns
        cache_np = cache_np.view(np.int16)
    cache = kvq.cache_from_canonical(torch.from_numpy(cache_np).cuda(), desc)
    scales = torch.from_numpy(scales_np).cuda()
    torch.cuda.synchronize()
    return cache, scales, desc

