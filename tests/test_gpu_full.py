"""GPU parity at the benchmark configurations' full sizes, in the launch configuration
bench.py times.  The library writes and attends over the whole workload; the CPU checker
writes and attends over a sample of sequences (it could do all of them, one by one, but
that takes minutes), and the two are compared on those: cache bytes and scales bit for bit,
attention within 2e-3 of the sampled output's max norm.  Every output must be finite."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_2605_29639_amd import workloads as W
from helpers import attn_err, gpu_attention, gpu_fill, oracle_fill

TOL = 2e-3


def sample_sequences(wl, extra=2):
    """Shortest, longest and a few more; sequence 0 first when a prefix is shared."""
    picks = {int(np.argmin(wl.seq_lens)), int(np.argmax(wl.seq_lens))}
    rng = np.random.default_rng(wl.seed + 99)
    while len(picks) < min(wl.batch, 2 + extra):
        picks.add(int(rng.integers(wl.batch)))
    if wl.shared_prefix:
        picks.add(0)
    return sorted(picks)


def compare_on_sample(wl, chunks, seqs=None):
    import torch
    from paper_2605_29639_amd import kvq
    seqs = sample_sequences(wl) if seqs is None else seqs
    cache, scales, desc = gpu_fill(wl)
    oc, osc = oracle_fill(wl, sequences=seqs)

    # --- the sampled sequences' blocks: codes and scales bit-exact ---
    bs = wl.block_size
    blocks = np.unique(np.concatenate(
        [wl.block_tables[b, :(int(wl.seq_lens[b]) + bs - 1) // bs] for b in seqs]))
    canon = kvq.cache_to_canonical(cache, desc)
    idx = torch.from_numpy(blocks.astype(np.int64)).cuda()
    got_c = canon[idx].cpu().numpy()
    if wl.mode == W.MODE_BF16:   # unquantized: bf16 bit patterns, no scales
        got_c = got_c.view(np.uint16)
    del canon
    bad = np.argwhere(got_c != oc[blocks])
    assert bad.size == 0, "codes differ, first at (sampled block, kv, h, off, d) %s" % bad[0]
    if wl.mode == W.MODE_FP8_TENSOR:
        assert np.array_equal(scales.cpu().numpy(), osc)
    elif wl.mode != W.MODE_BF16:
        got_s = scales[idx].cpu().numpy()
        assert np.array_equal(got_s.view(np.uint32), osc[blocks].view(np.uint32))

    # --- attention over everything on the GPU, over the sample on the CPU ---
    rows = np.concatenate([np.arange(b * wl.q_len, (b + 1) * wl.q_len) for b in seqs])
    want = oracle.paged_decode_attn(np.ascontiguousarray(wl.q[rows]), oc, osc, wl.mode,
                                    np.ascontiguousarray(wl.block_tables[seqs]),
                                    np.ascontiguousarray(wl.seq_lens[seqs]), wl.q_len,
                                    wl.sm_scale)
    errs = {}
    # (a workload with a shared prefix also goes through paged_decode_attn_prefix, as timed)
    for chunk in chunks:
        for prefix in sorted({0, wl.shared_prefix}):
            got = gpu_attention(wl, cache, scales, desc, chunk_tokens=chunk,
                                shared_prefix_tokens=prefix)
            assert np.isfinite(got).all(), "non-finite output (chunk %d)" % chunk
            errs[chunk, prefix] = attn_err(got[rows], want)
            assert errs[chunk, prefix] <= TOL, "chunk %d prefix %d: err %.3e on sequences %s" % (
                chunk, prefix, errs[chunk, prefix], seqs)
    return errs


def test_llama3_8b_layer_all_sequences():
    """Configuration 2 in full: the checker covers every sequence here."""
    wl = W.llama8b()
    assert wl.batch == 64 and 512 <= wl.seq_lens.min() and wl.seq_lens.max() <= 4096
    compare_on_sample(wl, chunks=(0, 512), seqs=list(range(wl.batch)))


def test_fp8_append_full_size():
    """Configuration 3: fp8 per block-head, cache built by bulk calls, then one appended token
    per sequence in a single call (block scales may grow and re-encode), then attention."""
    wl = W.fp8_append()
    assert wl.batch == 256 and wl.mode == W.MODE_FP8 and wl.append_tokens == 1
    compare_on_sample(wl, chunks=(0,))


def test_long_context_wide_gqa_full_size():
    """Configuration 4: G = 16, block 64, 16k-64k tokens, split-K over 2048-token ranges (the
    configuration's) and the automatic even split."""
    wl = W.long_gqa()
    assert wl.batch == 32 and wl.group == 16 and wl.chunk_tokens == 2048
    assert 16384 <= wl.seq_lens.min() and wl.seq_lens.max() <= 65536
    compare_on_sample(wl, chunks=(2048, 0), seqs=sample_sequences(wl, extra=1))


def test_unquantized_baseline_full_size():
    """The bf16 twin bench.py times beside the quantized path: configuration 2's shapes over an
    unquantized cache, and configuration 5's (two row tiles)."""
    wl = W.llama8b(mode=W.MODE_BF16)
    compare_on_sample(wl, chunks=(0,), seqs=sample_sequences(wl, extra=4))
    wl = W.verify_prefix(mode=W.MODE_BF16)
    compare_on_sample(wl, chunks=(0,), seqs=sample_sequences(wl, extra=0))


@pytest.mark.parametrize("mode", [W.MODE_INT4, W.MODE_INT4_GROUP, W.MODE_FP8_TENSOR])
def test_other_formats_full_size(mode):
    """Configuration 2's shapes with int4 per token-head codes and with e4m3 codes under static
    per-tensor scales."""
    wl = W.llama8b(mode=mode)
    compare_on_sample(wl, chunks=(0,), seqs=sample_sequences(wl, extra=6))


@pytest.mark.parametrize("mode", [W.MODE_INT8, W.MODE_FP8])
def test_verify_prefix_full_size(mode):
    """Configuration 5: 4 causal query tokens, G = 8 (32 query rows per kv head), the first
    1024 positions' blocks shared by all sequences; even layers int8, odd layers fp8."""
    wl = W.verify_prefix(mode=mode)
    assert wl.batch == 128 and wl.q_len == 4 and wl.group == 8 and wl.shared_prefix == 1024
    assert np.all(wl.block_tables[:, :64] == wl.block_tables[0, :64])
    compare_on_sample(wl, chunks=(0,), seqs=sample_sequences(wl, extra=1))


@pytest.mark.parametrize("mode", [W.MODE_INT8, W.MODE_FP8, W.MODE_BF16, W.MODE_INT4])
def test_chunk_prefill_full_size(mode):
    """The chunked-prefill shape bench.py times (8 sequences, 512 query tokens each over a
    4096-token prefix and themselves, 2048 query rows per kv head): every row of one sequence
    against the checker, the rest finite."""
    wl = W.chunk_prefill(mode)
    assert wl.batch == 8 and wl.q_len == 512 and int(wl.seq_lens[0]) == 4608
    compare_on_sample(wl, chunks=(0,), seqs=[5])
