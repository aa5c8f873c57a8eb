"""GPU parity, paged_decode_attn: within 2e-3 of the output's max norm of the CPU checker,
both reading the same quantized bytes (the checker's cache, uploaded)."""
import zlib

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_2605_29639_amd import workloads as W
from helpers import (attn_err, gpu_attention, gpu_fill, oracle_fill, upload_oracle_cache)

TOL = 2e-3   # max |gpu - oracle| <= TOL * max |oracle| over the call's whole output


def oracle_out(wl, oc, osc, seq_lens=None, q=None, q_len=None):
    return oracle.paged_decode_attn(wl.q if q is None else q, oc, osc, wl.mode, wl.block_tables,
                                    wl.seq_lens if seq_lens is None else seq_lens,
                                    wl.q_len if q_len is None else q_len, wl.sm_scale)


def check(wl, chunks=(0,), tol=TOL):
    oc, osc = oracle_fill(wl)
    want = oracle_out(wl, oc, osc)
    cache, scales, desc = upload_oracle_cache(wl, oc, osc)
    errs = []
    for chunk in chunks:
        got = gpu_attention(wl, cache, scales, desc, chunk_tokens=chunk)
        assert np.isfinite(got).all(), "non-finite output (chunk %d)" % chunk
        e = attn_err(got, want)
        errs.append(e)
        assert e <= tol, "chunk %d: err %.3e" % (chunk, e)
    return errs


MODES = [W.MODE_INT8, W.MODE_FP8, W.MODE_BF16, W.MODE_FP8_TENSOR, W.MODE_INT4, W.MODE_INT4_GROUP]


def skip_unsupported(mode, D):
    if mode in (W.MODE_INT4, W.MODE_INT4_GROUP) and D != 128:
        pytest.skip("int4 takes head_dim 128 only")


@pytest.mark.parametrize("mode", MODES)
def test_tiny_config(mode):
    skip_unsupported(mode, 64)
    check(W.tiny(mode), chunks=(0, 64))


CASES = [
    # name, seq_lens, q_len, Hq, Hkv, D, bs
    ("ragged16", [1, 15, 16, 17, 63, 64, 65, 255, 256, 257, 700], 1, 4, 2, 64, 16),
    ("d128_g4", [130, 333, 64, 1000, 5], 1, 32, 8, 128, 16),
    ("g1", [100, 260], 1, 2, 2, 128, 16),
    ("g2", [100, 260], 1, 4, 2, 64, 16),
    ("g8", [90, 515], 1, 16, 2, 128, 16),
    ("g16_bs64", [300, 1029, 64, 2049], 1, 64, 4, 128, 64),
    ("bs32", [257, 33], 1, 8, 2, 64, 32),
    ("bs128", [513, 100], 1, 8, 2, 128, 128),
    ("qlen4_g8", [53, 20, 4, 300, 1025], 4, 16, 2, 128, 16),
    ("qlen4_g4", [260, 7], 4, 8, 2, 64, 16),
    ("qlen2_g16", [100, 400], 2, 32, 2, 128, 64),
    ("qlen3_g16_rowgroups", [100, 130], 3, 32, 2, 64, 16),
    ("qlen16_g4", [100, 16, 77], 16, 4, 1, 128, 16),
    ("bs256", [700, 300, 256], 1, 8, 2, 128, 256),
    ("g64_two_row_groups", [150, 90], 1, 64, 1, 64, 16),
    ("qlen16_g8_four_row_groups", [200, 40], 16, 8, 1, 128, 32),
    # a chunk of a prompt attending over the quantized prefix and itself (causal)
    ("chunk64", [200, 70], 64, 8, 2, 128, 16),
    ("chunk200_bs64", [700], 200, 4, 1, 64, 64),
    ("chunk256", [300, 1029], 256, 16, 2, 128, 16),
    ("chunk40_ragged_row_block", [300, 41], 40, 8, 2, 128, 16),       # 160 rows: 128 + 32
    ("prompt_from_an_empty_cache", [130, 130], 130, 4, 1, 128, 16),    # q_len = the whole sequence
    ("chunk512_bs64_d64", [600, 512], 512, 8, 2, 64, 64),
    ("chunk96_g2_bs256", [700, 300], 96, 4, 2, 128, 256),              # 192 rows, 256-token blocks
    ("chunk130_g1_bs32_d64", [257, 140], 130, 2, 2, 64, 32),           # 130 rows: 128 + 2
    ("chunk140_g2_eight_pairs", [300, 140, 200, 141], 140, 4, 2, 64, 16),  # 8 (seq, head) pairs x 3 row blocks
]


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_shapes_and_splits(mode, case):
    name, lens, q_len, Hq, Hkv, D, bs = case
    skip_unsupported(mode, D)
    lens = [max(l, q_len) for l in lens]
    wl = W.custom(name, mode, lens, q_len, Hq, Hkv, D, bs, seed=zlib.crc32(name.encode()) % 1000 + mode)
    check(wl, chunks=(0, 64, 256))


@pytest.mark.parametrize("mode", MODES)
def test_gpu_written_cache_gives_the_same_attention(mode):
    """End to end through both entry points: the library's own cache (bit-identical to the
    checker's, see test_gpu_write) and the uploaded checker's cache give the same output."""
    wl = W.custom("e2e", mode, [200, 77, 1030], 1, 8, 2, 128, 16, seed=12)
    oc, osc = oracle_fill(wl)
    want = oracle_out(wl, oc, osc)
    c1, s1, desc = gpu_fill(wl)
    c2, s2, _ = upload_oracle_cache(wl, oc, osc)
    a = gpu_attention(wl, c1, s1, desc)
    b = gpu_attention(wl, c2, s2, desc)
    assert np.array_equal(a, b)
    assert attn_err(a, want) <= TOL


@pytest.mark.parametrize("q_len", [1, 40])   # 40 tokens x 4 heads: the many-row kernel
@pytest.mark.parametrize("mode", MODES)
def test_stale_bytes_after_the_last_position_are_never_used(mode, q_len):
    """Unwritten slots hold NaN codes / NaN or huge scales; block-table entries past the last
    block are -1.  The output must not change and must stay finite."""
    import torch
    D = 128 if mode in (W.MODE_INT4, W.MODE_INT4_GROUP) else 64
    lens = [max(l, q_len) for l in (37, 100, 64, 3)]
    wl = W.custom("stale", mode, lens, q_len, 4 if q_len == 1 else 8, 2, D, 16, seed=8)
    oc, osc = oracle_fill(wl)
    want = oracle_out(wl, oc, osc)
    live = np.zeros(oc.shape[:1] + oc.shape[3:4], dtype=bool)       # [blk, off]
    for b in range(wl.batch):
        s = wl.slots(b, 0, int(wl.seq_lens[b]))
        live[s // 16, s % 16] = True
    dirty_c, dirty_s = oc.copy(), osc.copy()
    for blk, off in np.argwhere(~live):
        if mode == W.MODE_BF16:   # NaN and infinity bit patterns
            dirty_c[blk, :, :, off, :] = 0x7FC0 if (blk + off) % 2 else 0xFF80
        else:
            dirty_c[blk, :, :, off, :] = 0x80 if mode == W.MODE_INT8 else 0x7F
        if mode in (W.MODE_INT8, W.MODE_INT4, W.MODE_INT4_GROUP):
            dirty_s[blk, :, :, off] = np.nan if (blk + off) % 2 else 3e38
    if mode == W.MODE_FP8:
        dead_blocks = ~live.any(axis=1)
        dirty_s[dead_blocks] = np.nan
    cache, scales, desc = upload_oracle_cache(wl, dirty_c, dirty_s)
    for chunk in (0, 64):
        got = gpu_attention(wl, cache, scales, desc, chunk_tokens=chunk)
        assert np.isfinite(got).all()
        assert attn_err(got, want) <= TOL


def test_run_to_run_determinism():
    wl = W.custom("det", W.MODE_INT8, [900, 333], 1, 8, 2, 128, 16, seed=2)
    cache, scales, desc = gpu_fill(wl)
    a = gpu_attention(wl, cache, scales, desc, chunk_tokens=256)
    b = gpu_attention(wl, cache, scales, desc, chunk_tokens=256)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("mode", MODES[:3])  # (one static scale cannot span these magnitudes)
def test_degenerate_inputs(mode):
    """All-zero V rows carrying the largest weight, zero q, huge and tiny V magnitudes."""
    wl = W.custom("degenerate", mode, [80, 80, 80, 80], 1, 4, 2, 64, 16, seed=21, outliers=False)
    oc, osc = oracle.alloc_cache(mode, wl.num_blocks, 16, 2, 64)
    for b in range(4):
        k, v = wl.kv_rows(b, 0, 80)
        kf, vf = W.bf16_bits_to_f32(k), W.bf16_bits_to_f32(v)
        if b == 0:      # an "attention sink": strongest key, zero value
            kf[0, :] = W.bf16_bits_to_f32(wl.q[0]).reshape(2, 2, 64)[:, 0] * 3
            vf[0] = 0
        if b == 1:      # zero query
            wl.q[1] = 0
        if b == 2:      # V spans 40 binades across tokens
            vf *= (2.0 ** np.linspace(-20, 20, 80)).astype(np.float32)[:, None, None]
        if b == 3:      # everything tiny
            vf *= np.float32(2.0 ** -60)
            kf *= np.float32(2.0 ** -30)
        oracle.kv_quant_write(W.to_bf16_bits(kf), W.to_bf16_bits(vf), wl.slots(b, 0, 80), oc, osc,
                              mode)
    want = oracle_out(wl, oc, osc)
    cache, scales, desc = upload_oracle_cache(wl, oc, osc)
    got = gpu_attention(wl, cache, scales, desc)
    assert np.isfinite(got).all()
    for b in range(4):   # per sequence, since their magnitudes differ by design
        assert attn_err(got[b], want[b]) <= TOL, b


def test_empty_batch():
    import torch
    from paper_2605_29639_amd import kvq
    desc = kvq.make_desc(0, 4, 16, 2, 64)
    cache, scales = kvq.alloc_cache(desc)
    q = torch.empty((0, 4, 64), dtype=torch.bfloat16, device="cuda")
    out = torch.empty((0, 4, 64), dtype=torch.float32, device="cuda")
    ws = torch.empty(16, dtype=torch.uint8, device="cuda")
    kvq.paged_decode_attn(q, cache, scales, desc,
                          torch.empty((0, 4), dtype=torch.int32, device="cuda"),
                          torch.empty(0, dtype=torch.int32, device="cuda"), 1, 0, 0.125, out, ws)
    torch.cuda.synchronize()


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes(seed):
    """Shapes nobody picked by hand: batch, lengths, group size, query tokens, block size, head
    size, cache mode and split granule all drawn from a seeded generator."""
    rng = np.random.default_rng(7000 + seed)
    D = int(rng.choice([64, 128]))
    modes = [m for m in MODES if not (m in (W.MODE_INT4, W.MODE_INT4_GROUP) and D != 128)]
    mode = int(rng.choice(modes))
    bs = int(rng.choice([16, 32, 64, 128]))
    Hkv = int(rng.choice([1, 2, 3]))
    G = int(rng.choice([1, 2, 4, 8, 16]))
    q_len = int(rng.choice([1, 1, 2, 3, 4, 8]))
    B = int(rng.integers(1, 10))
    lens = [int(rng.choice([rng.integers(q_len, 70), rng.integers(q_len, 1500),
                            64 * rng.integers(1, 9)])) for _ in range(B)]
    lens = [max(l, q_len) for l in lens]
    chunk = int(rng.choice([0, 64, 128, 512]))
    wl = W.custom("random%d" % seed, mode, lens, q_len, G * Hkv, Hkv, D, bs, seed=seed)
    check(wl, chunks=(chunk,))


@pytest.mark.parametrize("mode,q_len,prefix,batch,spread",
                         [(W.MODE_INT8, 1, 0, 3000, 200), (W.MODE_FP8, 1, 0, 1500, 200),
                          (W.MODE_INT8, 4, 0, 3000, 200), (W.MODE_BF16, 1, 0, 3000, 200),
                          (W.MODE_INT8, 2, 256, 2000, 100), (W.MODE_FP8, 4, 256, 1100, 64)])
def test_thousands_of_short_sequences(mode, q_len, prefix, batch, spread):
    """Far more (sequence, kv head) pairs than wavefronts: every range of the flat list crosses
    many pairs, most pairs lie inside one range and are written without a partial, and the
    per-sequence bookkeeping (lengths, prefix sums) runs over a batch many times the
    wavefront's width.  With a prefix: the same through the shared-prefix entry point."""
    rng = np.random.default_rng(900 + q_len)
    lo = max(q_len, prefix)
    lens = [int(x) for x in rng.integers(lo, lo + spread, size=batch)]
    lens[17] = lo              # the shortest allowed
    lens[batch - 1] = lo + 700  # and a long one at the very end of the list
    wl = W.custom("crowd", mode, lens, q_len, 4, 2, 128, 16, seed=77, shared_prefix=prefix)
    oc, osc = oracle_fill(wl)
    want = oracle_out(wl, oc, osc)
    cache, scales, desc = upload_oracle_cache(wl, oc, osc)
    for hint in ((0,) if prefix == 0 else (prefix, 64, 0)):
        got = gpu_attention(wl, cache, scales, desc, chunk_tokens=0, shared_prefix_tokens=hint)
        assert np.isfinite(got).all()
        e = attn_err(got, want)
        assert e <= TOL, "shared_prefix_tokens %d: err %.3e" % (hint, e)


@pytest.mark.parametrize("mode,D", [(W.MODE_INT8, 128), (W.MODE_FP8, 64), (W.MODE_BF16, 128),
                                    (W.MODE_INT4_GROUP, 128)])
def test_the_largest_query_length(mode, D):
    """q_len at the library's limit (1024 query tokens per sequence): a whole prompt of exactly
    that length, and a chunk of that length over a shorter prefix."""
    wl = W.custom("longest_chunk", mode, [1024, 1500], 1024, 4, 2, D, 16, seed=31 + mode)
    check(wl)


@pytest.mark.parametrize("mode", MODES)
def test_many_query_rows_through_both_kernels(mode):
    """128 and more query rows per kv head take the kernel that shares the dequantization among
    128 rows; the streaming kernels must give the same answer (both within the bound of the
    checker, and close to each other)."""
    from paper_2605_29639_amd import kvq
    wl = W.custom("both", mode, [700, 129, 64], 64, 8, 2, 128, 16, seed=40 + mode)
    oc, osc = oracle_fill(wl)
    want = oracle_out(wl, oc, osc)
    cache, scales, desc = upload_oracle_cache(wl, oc, osc)
    shared = gpu_attention(wl, cache, scales, desc)
    prof = kvq.prof_lib()   # the measurement build can keep such calls on the streaming kernels
    prof.kvq_profile_prefill_kernel(0)
    try:
        streamed = gpu_attention(wl, cache, scales, desc, L=prof)
    finally:
        prof.kvq_profile_prefill_kernel(1)
    assert attn_err(shared, want) <= TOL and attn_err(streamed, want) <= TOL
    assert attn_err(shared, streamed.astype(np.float64)) <= 2e-4


PREFIX_LENS = {
    "ragged": [700, 256, 1500, 333, 257],       # one sequence is nothing but the prefix
    "one": [1000],                              # a single pair per kv head
    "many": [256 + 37 * (i % 9) for i in range(70)],   # more sequences than a wavefront has lanes
}


@pytest.mark.parametrize("mode", [W.MODE_INT8, W.MODE_FP8, W.MODE_BF16, W.MODE_INT4])
@pytest.mark.parametrize("q_len", [1, 4])
@pytest.mark.parametrize("lens", sorted(PREFIX_LENS))
def test_shared_prefix_is_read_through_stacked_rows(mode, q_len, lens):
    """paged_decode_attn_prefix: sequences that begin with the same physical blocks.  The
    shared positions go through the many-row kernel with all sequences' rows stacked, the rest
    through the streaming kernel, and the reduce merges the two: the output stays within the
    bound of the checker and close to paged_decode_attn's (other order of the fp32 merges; the
    probabilities are rounded to 16 bits against a running maximum that depends on the order),
    also with ranges given by chunk_tokens, with a prefix that is not a multiple of 64, with a
    sequence that is nothing but the prefix (its query rows then mask part of it) and with more
    sequences than a wavefront has lanes.  A prefix longer than the shortest sequence is dropped
    (on the host if it exceeds max_seq_len, else on the device), as is one below 64 tokens or
    with a single sequence: bit for bit paged_decode_attn's output then."""
    wl = W.custom("prefix", mode, PREFIX_LENS[lens], q_len, 8, 2, 128, 16,
                  seed=90 + mode + q_len, shared_prefix=256)
    assert (wl.block_tables[:, :16] == wl.block_tables[0, :16]).all()
    oc, osc = oracle_fill(wl)
    want = oracle_out(wl, oc, osc)
    cache, scales, desc = upload_oracle_cache(wl, oc, osc)
    shortest = min(PREFIX_LENS[lens])
    for chunk in (0, 128, 512):
        plain = gpu_attention(wl, cache, scales, desc, chunk_tokens=chunk)
        assert attn_err(plain, want) <= TOL
        for hint in (256, 200, 64, 63, 4096) + ((shortest + 64,) if lens != "one" else ()):
            hinted = gpu_attention(wl, cache, scales, desc, chunk_tokens=chunk,
                                   shared_prefix_tokens=hint)
            used = 64 <= hint and hint // 64 * 64 <= shortest and len(PREFIX_LENS[lens]) > 1
            if not used:
                assert np.array_equal(hinted.view(np.uint32), plain.view(np.uint32)), hint
            else:
                assert attn_err(hinted, want) <= TOL, (chunk, hint)
                assert attn_err(hinted, plain.astype(np.float64)) <= 2e-4, (chunk, hint)
