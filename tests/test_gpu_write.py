"""GPU parity, kv_quant_write: codes, scales and slot indexing must equal the CPU checker's
bit for bit, over the whole pool (both sides start from a zero-filled pool)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_2605_29639_amd import workloads as W
from helpers import bits_to_bf16_tensor, gpu_desc, gpu_fill, oracle_fill


ALL_MODES = [W.MODE_INT8, W.MODE_FP8, W.MODE_BF16, W.MODE_FP8_TENSOR, W.MODE_INT4, W.MODE_INT4_GROUP]


def skip_unsupported(mode, D):
    if mode in (W.MODE_INT4, W.MODE_INT4_GROUP) and D != 128:
        pytest.skip("int4 takes head_dim 128 only")


def fetch(cache, scales, desc):
    from paper_2605_29639_amd import kvq
    canon = kvq.cache_to_canonical(cache, desc).cpu().numpy()
    if canon.dtype == np.int16:  # unquantized cache: bf16 bit patterns
        canon = canon.view(np.uint16)
    return canon, scales.cpu().numpy()


def assert_pool_equal(wl, got, want):
    (gc, gs), (wc, ws) = got, want
    assert gc.shape == wc.shape and gs.shape == ws.shape
    bad = np.argwhere(gc != wc)
    assert bad.size == 0, "codes differ at (blk,kv,h,off,d) %s: gpu %s oracle %s (%d total)" % (
        bad[0], gc[tuple(bad[0])], wc[tuple(bad[0])], len(bad))
    sb = np.argwhere(gs.view(np.uint32) != ws.view(np.uint32))
    assert sb.size == 0, "scales differ at %s: gpu %r oracle %r" % (
        sb[0], gs[tuple(sb[0])], ws[tuple(sb[0])])


@pytest.mark.parametrize("mode", ALL_MODES)
def test_tiny_config(mode):
    skip_unsupported(mode, 64)
    wl = W.tiny(mode)
    cache, scales, desc = gpu_fill(wl)
    assert_pool_equal(wl, fetch(cache, scales, desc), oracle_fill(wl))


SHAPES = [
    # seq_lens, H_kv, D, bs
    ([1, 15, 16, 17, 31, 32, 33, 200], 2, 64, 16),
    ([130, 64, 65, 63, 1], 3, 128, 16),
    ([300, 129, 64], 2, 128, 64),
    ([257, 5], 1, 64, 32),
    ([513], 4, 128, 128),
    ([700, 300], 2, 128, 256),
]


@pytest.mark.parametrize("mode", ALL_MODES)
@pytest.mark.parametrize("shape", SHAPES)
def test_ragged_shapes_bulk_write(mode, shape):
    lens, H, D, bs = shape
    skip_unsupported(mode, D)
    wl = W.custom("ragged", mode, lens, 1, H * 2, H, D, bs, seed=1000 + D + bs + mode)
    cache, scales, desc = gpu_fill(wl)
    assert_pool_equal(wl, fetch(cache, scales, desc), oracle_fill(wl))


@pytest.mark.parametrize("mode", [W.MODE_INT8, W.MODE_FP8, W.MODE_FP8_TENSOR, W.MODE_INT4,
                                  W.MODE_INT4_GROUP])
@pytest.mark.parametrize("bs,D,H", [(16, 128, 2), (64, 64, 3), (32, 128, 1), (256, 128, 1), (128, 64, 2)])
def test_prefill_of_several_sequences_in_one_call(mode, bs, D, H):
    """Thousands of tokens in one call (the prefill kernels): ragged sequences back to back, so
    that runs start at any token index; one sequence continued from the middle of a block;
    skipped tokens; rows full of rounding ties, tiny and huge rows."""
    import torch
    from paper_2605_29639_amd import kvq
    skip_unsupported(mode, D)
    lens = [700, 33, 1, 1234, 16, 515, 47]
    wl = W.custom("prefill", mode, lens, 1, H, H, D, bs, seed=31 + bs + D + mode)
    desc = gpu_desc(wl)
    cache, scales = kvq.alloc_cache(desc)
    oc, osc = oracle.alloc_cache(mode, wl.num_blocks, bs, H, D)
    if mode == W.MODE_FP8_TENSOR:
        osc[:] = W.STATIC_SCALES
        scales.copy_(torch.from_numpy(osc))
    # sequence 3's first 21 tokens were written by an earlier call
    k, v = wl.kv_rows(3, 0, 21)
    s = wl.slots(3, 0, 21)
    oracle.kv_quant_write(k, v, s, oc, osc, mode)
    kvq.kv_quant_write(bits_to_bf16_tensor(k), bits_to_bf16_tensor(v), torch.from_numpy(s).cuda(),
                       cache, scales, desc)
    ks, vs, ss = [], [], []
    for b, L in enumerate(lens):
        lo = 21 if b == 3 else 0
        k, v = wl.kv_rows(b, lo, L)
        kf, vf = W.bf16_bits_to_f32(k), W.bf16_bits_to_f32(v)
        if b == 0:
            qmax = {W.MODE_INT8: 127.0, W.MODE_INT4: 7.0, W.MODE_INT4_GROUP: 7.0}.get(mode, 448.0)
            vf[64:128] = np.round(vf[64:128] * 16) / 2   # half-integers ...
            vf[64:128, :, 0] = qmax                      # ... at scale exactly 1: ties
            kf[128:160] *= np.float32(2.0 ** -120)       # scales below the normal fp32 range
            kf[160:192] *= np.float32(2.0 ** 110)
            kf[200:216] = 0
        s = wl.slots(b, lo, L)
        if b == 5:
            s[-3:] = -1                                  # skipped tokens at a run's end
        ks.append(W.to_bf16_bits(kf)), vs.append(W.to_bf16_bits(vf)), ss.append(s)
    k, v, s = np.concatenate(ks), np.concatenate(vs), np.concatenate(ss)
    assert len(s) >= 2048
    oracle.kv_quant_write(k, v, s, oc, osc, mode)
    kvq.kv_quant_write(bits_to_bf16_tensor(k), bits_to_bf16_tensor(v), torch.from_numpy(s).cuda(),
                       cache, scales, desc)
    torch.cuda.synchronize()
    assert_pool_equal(wl, fetch(cache, scales, desc), (oc, osc))


@pytest.mark.parametrize("bs,D", [(16, 128), (64, 64)])
def test_fp8_token_by_token_append_with_rescale(bs, D):
    """Decode-style appends: each call adds one token per sequence; magnitudes vary so that the
    block scale grows several times and earlier codes are re-encoded."""
    import torch
    from paper_2605_29639_amd import kvq
    wl = W.custom("append", W.MODE_FP8, [40, 70, 19], 1, 4, 2, D, bs, seed=77)
    rng = np.random.default_rng(5)
    desc = gpu_desc(wl)
    cache, scales = kvq.alloc_cache(desc)
    oc, osc = oracle.alloc_cache(wl.mode, wl.num_blocks, bs, 2, D)
    rows = {b: wl.kv_rows(b, 0, int(wl.seq_lens[b])) for b in range(wl.batch)}
    gain = {b: rng.choice([0.05, 0.3, 1.0, 4.0, 30.0], size=int(wl.seq_lens[b])) for b in range(3)}
    for step in range(int(wl.seq_lens.max())):
        ks, vs, ss = [], [], []
        for b in range(wl.batch):
            if step < wl.seq_lens[b]:
                k = W.to_bf16_bits(W.bf16_bits_to_f32(rows[b][0][step:step + 1]) * np.float32(gain[b][step]))
                v = W.to_bf16_bits(W.bf16_bits_to_f32(rows[b][1][step:step + 1]) * np.float32(gain[b][step]))
                ks.append(k), vs.append(v), ss.append(wl.slots(b, step, step + 1))
        k, v, s = np.concatenate(ks), np.concatenate(vs), np.concatenate(ss)
        oracle.kv_quant_write(k, v, s, oc, osc, wl.mode)
        kvq.kv_quant_write(bits_to_bf16_tensor(k), bits_to_bf16_tensor(v),
                           torch.from_numpy(s).cuda(), cache, scales, desc)
    torch.cuda.synchronize()
    assert_pool_equal(wl, fetch(cache, scales, desc), (oc, osc))


@pytest.mark.parametrize("mode", ALL_MODES)
def test_chunked_prefill_then_appends(mode):
    """A sequence written in uneven pieces (block-aligned or not) and then appended to."""
    import torch
    from paper_2605_29639_amd import kvq
    wl = W.custom("pieces", mode, [150], 1, 4, 2, 128, 16, seed=9)
    desc = gpu_desc(wl)
    cache, scales = kvq.alloc_cache(desc)
    oc, osc = oracle.alloc_cache(mode, wl.num_blocks, 16, 2, 128)
    if mode == W.MODE_FP8_TENSOR:
        osc[:] = W.STATIC_SCALES
        scales.copy_(torch.from_numpy(osc))
    for lo, hi in ((0, 16), (16, 37), (37, 38), (38, 96), (96, 149), (149, 150)):
        k, v = wl.kv_rows(0, lo, hi)
        s = wl.slots(0, lo, hi)
        oracle.kv_quant_write(k, v, s, oc, osc, mode)
        kvq.kv_quant_write(bits_to_bf16_tensor(k), bits_to_bf16_tensor(v),
                           torch.from_numpy(s).cuda(), cache, scales, desc)
    torch.cuda.synchronize()
    assert_pool_equal(wl, fetch(cache, scales, desc), (oc, osc))


@pytest.mark.parametrize("mode", [W.MODE_INT8, W.MODE_FP8, W.MODE_INT4, W.MODE_INT4_GROUP])
def test_zero_rows_negative_zero_skipped_tokens_and_stale_pool(mode):
    import torch
    from paper_2605_29639_amd import kvq
    D = 128 if mode in (W.MODE_INT4, W.MODE_INT4_GROUP) else 64
    wl = W.custom("edge", mode, [48], 1, 2, 2, D, 16, seed=3)
    k, v = wl.kv_rows(0, 0, 48)
    k[3] = 0                     # all-zero K row (both heads)
    v[3, 0] = 0x8000             # all negative-zero V row for head 0
    k[16:32, 1] = 0              # a whole block of zeros for head 1 (fp8: block scale 0)
    v[40, :, :] = 0
    v[40, 0, 5] = 0x8000
    slots = wl.slots(0, 0, 48)
    # skipped tokens: for the block-scaled fp8 cache at the end of a block's run (its tokens of
    # one call must be one run of consecutive slots per block), anywhere for the other formats
    slots[15 if mode == W.MODE_FP8 else 7] = -1
    slots[47 if mode == W.MODE_FP8 else 41] = -1
    desc = gpu_desc(wl)
    # stale pool on both sides: NaN codes and a garbage scale everywhere
    oc, osc = oracle.alloc_cache(mode, wl.num_blocks, 16, 2, D)
    oc[:] = 0x7F
    osc[:] = 123.0
    cache = kvq.cache_from_canonical(torch.from_numpy(oc).cuda(), desc)
    scales = torch.from_numpy(osc).cuda()
    oracle.kv_quant_write(k, v, slots, oc, osc, mode)
    kvq.kv_quant_write(bits_to_bf16_tensor(k), bits_to_bf16_tensor(v),
                       torch.from_numpy(slots).cuda(), cache, scales, desc)
    torch.cuda.synchronize()
    assert_pool_equal(wl, fetch(cache, scales, desc), (oc, osc))


def test_extreme_magnitudes_int8_and_fp8():
    """Rows near the top and bottom of the bf16 range, and values that land on rounding ties."""
    import torch
    from paper_2605_29639_amd import kvq
    for mode in (W.MODE_INT8, W.MODE_FP8):
        wl = W.custom("extreme", mode, [64], 1, 1, 1, 128, 16, seed=4, outliers=False)
        k, v = wl.kv_rows(0, 0, 64)
        kf, vf = W.bf16_bits_to_f32(k), W.bf16_bits_to_f32(v)
        kf[0:16] *= np.float32(2.0 ** 100)
        kf[16:32] *= np.float32(2.0 ** -110)
        vf[0:16] = np.round(vf[0:16] * 16) / 2          # half-integers
        vf[0:16, 0, 0] = 127.0 if mode == 0 else 448.0  # scale exactly 1: ties everywhere
        vf[16:32] = np.round(vf[16:32] * 64) / 64
        vf[16:32, 0, 1] = 254.0 if mode == 0 else 224.0
        k, v = W.to_bf16_bits(kf), W.to_bf16_bits(vf)
        desc = gpu_desc(wl)
        cache, scales = kvq.alloc_cache(desc)
        oc, osc = oracle.alloc_cache(mode, wl.num_blocks, 16, 1, 128)
        s = wl.slots(0, 0, 64)
        oracle.kv_quant_write(k, v, s, oc, osc, mode)
        kvq.kv_quant_write(bits_to_bf16_tensor(k), bits_to_bf16_tensor(v),
                           torch.from_numpy(s).cuda(), cache, scales, desc)
        torch.cuda.synchronize()
        assert_pool_equal(wl, fetch(cache, scales, desc), (oc, osc))


def test_repack_round_trip_and_layout():
    """to_canonical(from_canonical(x)) = x, and the physical layout is the documented one:
    K in 4-token quads of 16-channel slices, V channel-major per 16-token sub-block, int8
    codes stored as code XOR 0x80."""
    import torch
    from paper_2605_29639_amd import kvq
    nblk, bs, H, D = 5, 32, 3, 64
    desc = kvq.make_desc(0, nblk, bs, H, D)
    rng = np.random.default_rng(0)
    canon = rng.integers(0, 256, size=desc.cache_shape(), dtype=np.uint8)
    phys = kvq.cache_from_canonical(torch.from_numpy(canon).cuda(), desc)
    back = kvq.cache_to_canonical(phys, desc).cpu().numpy()
    assert np.array_equal(back, canon)
    p = phys.cpu().numpy().reshape(nblk, 2, H, bs * D)
    # K: [quad][slice][token in quad][16 channels]
    k = p[:, 0].reshape(nblk, H, bs // 4, D // 16, 4, 16)
    want_k = canon[:, 0].reshape(nblk, H, bs // 4, 4, D // 16, 16).transpose(0, 1, 2, 4, 3, 5)
    assert np.array_equal(k, want_k ^ 0x80)
    # V: [sub-block][channel][16 tokens]
    v = p[:, 1].reshape(nblk, H, bs // 16, D, 16)
    want_v = canon[:, 1].reshape(nblk, H, bs // 16, 16, D).transpose(0, 1, 2, 4, 3)
    assert np.array_equal(v, want_v ^ 0x80)
    # e4m3 codes are stored as they are
    desc8 = kvq.make_desc(1, nblk, bs, H, D)
    phys8 = kvq.cache_from_canonical(torch.from_numpy(canon).cuda(), desc8)
    assert np.array_equal(phys8.cpu().numpy(), phys.cpu().numpy() ^ 0x80)
    assert np.array_equal(kvq.cache_to_canonical(phys8, desc8).cpu().numpy(), canon)


def test_empty_write_is_a_no_op():
    import torch
    from paper_2605_29639_amd import kvq
    desc = kvq.make_desc(1, 4, 16, 2, 64)
    cache, scales = kvq.alloc_cache(desc)
    k = torch.empty((0, 2, 64), dtype=torch.bfloat16, device="cuda")
    kvq.kv_quant_write(k, k, torch.empty(0, dtype=torch.int64, device="cuda"), cache, scales, desc)
    torch.cuda.synchronize()
    assert not cache.any() and not scales.any()


def random_segments(rng, num_tokens, nblk, bs):
    """slot_mapping of about num_tokens tokens: runs of consecutive slots of random length that
    start anywhere inside a block, each block touched by at most one run, the runs in random
    token order with skipped tokens (-1) sprinkled between them."""
    segments, blk, total = [], 0, 0
    while total < num_tokens and blk < nblk - 8:
        off = int(rng.integers(0, bs))
        length = int(rng.integers(1, 3 * bs + 1))
        if rng.random() < 0.3:
            off, length = 0, bs * int(rng.integers(1, 5))      # whole blocks, as a prompt writes
        first = blk * bs + off
        segments.append(np.arange(first, first + length, dtype=np.int64))
        blk += (off + length + bs - 1) // bs + int(rng.integers(0, 3))
        total += length
    order = rng.permutation(len(segments))
    parts = []
    for i in order:
        parts.append(segments[i])
        if rng.random() < 0.25:
            parts.append(np.full(int(rng.integers(1, 4)), -1, dtype=np.int64))
    return np.concatenate(parts)


@pytest.mark.parametrize("mode", ALL_MODES)
@pytest.mark.parametrize("num_tokens", [60, 1700])       # per-run kernels, prefill kernels
@pytest.mark.parametrize("bs", [16, 64])
def test_random_slot_patterns(mode, num_tokens, bs):
    import torch
    from paper_2605_29639_amd import kvq
    H, D = 2, 128
    rng = np.random.default_rng(900 + 10 * mode + num_tokens + bs)
    nblk = num_tokens // bs * 3 + 40
    slots = random_segments(rng, num_tokens, nblk, bs)
    T = len(slots)
    x = (rng.standard_normal((2, T, H, D), dtype=np.float32) *
         rng.choice([0.01, 1.0, 30.0], size=(2, T, H, 1)).astype(np.float32))
    k, v = W.to_bf16_bits(x[0]), W.to_bf16_bits(x[1])
    desc = kvq.make_desc(mode, nblk, bs, H, D)
    cache, scales = kvq.alloc_cache(desc)
    oc, osc = oracle.alloc_cache(mode, nblk, bs, H, D)
    if mode == W.MODE_FP8_TENSOR:
        osc[:] = (0.07, 0.11)
        scales.copy_(torch.from_numpy(osc))
    oracle.kv_quant_write(k, v, slots, oc, osc, mode)
    kvq.kv_quant_write(bits_to_bf16_tensor(k), bits_to_bf16_tensor(v), torch.from_numpy(slots).cuda(),
                       cache, scales, desc)
    torch.cuda.synchronize()
    assert_pool_equal(None, fetch(cache, scales, desc), (oc, osc))


@pytest.mark.parametrize("mode", [W.MODE_INT8, W.MODE_BF16, W.MODE_FP8_TENSOR, W.MODE_INT4,
                                  W.MODE_INT4_GROUP])
@pytest.mark.parametrize("num_tokens", [150, 1500])      # per-run kernels, prefill kernels
@pytest.mark.parametrize("bs", [16, 64])
def test_tokens_in_any_order_with_skips_anywhere(mode, num_tokens, bs):
    """Every format but the block-scaled fp8 takes a call's tokens in any order: distinct slots
    in fully shuffled token order, so that almost every token is a run of its own and the
    tokens of one 16-token sub-block are handled by different wavefronts; skipped tokens (-1)
    anywhere; a stretch left in slot order with single tokens knocked out of it in mid
    sub-block; a stale pool underneath, so that a lost or misplaced update shows."""
    import torch
    from paper_2605_29639_amd import kvq
    H, D = 2, 128
    rng = np.random.default_rng(4100 + 10 * mode + num_tokens + bs)
    nblk = num_tokens // bs + 12
    # 3/4 of the pool's slots, shuffled; the last quarter of the tokens back in slot order
    slots = rng.permutation(nblk * bs)[: num_tokens].astype(np.int64)
    tail = num_tokens // 4
    slots[-tail:] = np.sort(slots[-tail:])
    dense = np.arange(5 * bs, 7 * bs, dtype=np.int64)     # two whole blocks in slot order ...
    slots = np.concatenate([slots[~np.isin(slots, dense)], dense])
    slots[-2 * bs + 5] = -1                               # ... with holes in mid sub-block
    slots[-bs + 9] = -1
    slots[rng.random(len(slots)) < 0.05] = -1
    T = len(slots)
    x = (rng.standard_normal((2, T, H, D), dtype=np.float32) *
         rng.choice([0.01, 1.0, 30.0], size=(2, T, H, 1)).astype(np.float32))
    k, v = W.to_bf16_bits(x[0]), W.to_bf16_bits(x[1])
    desc = kvq.make_desc(mode, nblk, bs, H, D)
    oc, osc = oracle.alloc_cache(mode, nblk, bs, H, D)
    oc[:] = 0x5A                                          # stale codes and scales on both sides
    osc[:] = (0.07, 0.11) if mode == W.MODE_FP8_TENSOR else 3.0
    canon = torch.from_numpy(oc.view(np.int16) if oc.dtype == np.uint16 else oc).cuda()
    cache = kvq.cache_from_canonical(canon, desc)
    scales = torch.from_numpy(osc).cuda()
    oracle.kv_quant_write(k, v, slots, oc, osc, mode)
    kvq.kv_quant_write(bits_to_bf16_tensor(k), bits_to_bf16_tensor(v), torch.from_numpy(slots).cuda(),
                       cache, scales, desc)
    torch.cuda.synchronize()
    assert_pool_equal(None, fetch(cache, scales, desc), (oc, osc))
