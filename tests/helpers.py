"""Shared by the tests: build an oracle-written cache for a workload (CPU only)."""
import numpy as np

import oracle


def oracle_fill(wl, sequences=None):
    """Zero pool, then the oracle writes every sequence's prefill rows (one call per
    sequence, all of its tokens at once) and, if the workload has an append step, one
    more call carrying the appended token of every sequence.  With `sequences`, only
    those sequences are written (the rest of the pool stays zero)."""
    cache, scales = oracle.alloc_cache(wl.mode, wl.num_blocks, wl.block_size, wl.num_kv_heads,
                                       wl.head_dim)
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
