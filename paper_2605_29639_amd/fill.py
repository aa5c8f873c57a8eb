"""Device-side plumbing shared by the benchmark, the smoke check and the tests: turning the
synthetic workloads' numpy arrays into device tensors and writing a workload into a cache
through the library's own kv_quant_write.  No arithmetic of the method lives here."""
import numpy as np

from . import workloads as W


def bits_to_bf16_tensor(bits, device="cuda"):
    """uint16 bf16 bit patterns (numpy) -> torch.bfloat16 device tensor (no value change)."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def gpu_desc(wl):
    from . import kvq
    return kvq.make_desc(wl.mode, wl.num_blocks, wl.block_size, wl.num_kv_heads, wl.head_dim)


def append_inputs(wl, sequences=None):
    """(k, v, slot_mapping) device tensors of the workload's append step: the last
    `append_tokens` positions of every sequence, sequence-major."""
    import torch
    ks, vs, ss = [], [], []
    for b in (range(wl.batch) if sequences is None else sequences):
        p0, p1 = wl.prefill_len(b), int(wl.seq_lens[b])
        k, v = wl.kv_rows(b, p0, p1)
        ks.append(k), vs.append(v), ss.append(wl.slots(b, p0, p1))
    return (bits_to_bf16_tensor(np.concatenate(ks)), bits_to_bf16_tensor(np.concatenate(vs)),
            torch.from_numpy(np.concatenate(ss)).cuda())


def gpu_fill(wl, sequences=None, cache=None, scales=None, workers=8):
    """The library writes the workload into a (zeroed unless given) device pool: one call per
    sequence carrying all of its prefill tokens, then, if the workload has an append step, one
    call carrying the appended tokens of every sequence.  Returns (cache, scales, desc).
    The rows are drawn on `workers` host threads ahead of the calls that consume them."""
    import torch
    from concurrent.futures import ThreadPoolExecutor
    from . import kvq
    desc = gpu_desc(wl)
    if cache is None:
        cache, scales = kvq.alloc_cache(desc)
        if wl.mode == W.MODE_FP8_TENSOR:
            scales.copy_(torch.tensor(W.STATIC_SCALES, dtype=torch.float32))
    seqs = [b for b in (range(wl.batch) if sequences is None else sequences)
            if wl.write_range(b)[1] > wl.write_range(b)[0]]

    def draw(b):
        start, stop = wl.write_range(b)
        k, v = wl.kv_rows(b, start, stop)
        return k, v, wl.slots(b, start, stop)

    with ThreadPoolExecutor(max_workers=max(1, workers)) as pool:
        ahead = 2 * max(1, workers)
        pending = [pool.submit(draw, b) for b in seqs[:ahead]]
        for i in range(len(seqs)):
            k, v, slots = pending[i].result()
            pending[i] = None
            if i + ahead < len(seqs):
                pending.append(pool.submit(draw, seqs[i + ahead]))
            kvq.kv_quant_write(bits_to_bf16_tensor(k), bits_to_bf16_tensor(v),
                               torch.from_numpy(slots).cuda(), cache, scales, desc)
    if wl.append_tokens:
        k, v, slots = append_inputs(wl, range(wl.batch) if sequences is None else sequences)
        kvq.kv_quant_write(k, v, slots, cache, scales, desc)
    torch.cuda.synchronize()
    return cache, scales, desc


def attn_err(got, want):
    """max |got - want| / max |want| over the whole output tensor."""
    return float(np.abs(got.astype(np.float64) - want).max() / np.abs(want).max())
