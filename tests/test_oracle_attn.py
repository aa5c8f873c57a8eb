"""Pins for the CPU checker's attention half (CPU only): closed forms, invariants, special
cases and an independent dense brute force.  No expected value comes from the checker's own
attention loops."""
import numpy as np
import pytest

import oracle
from oracle import brute
from paper_2605_29639_amd import workloads as W
from helpers import oracle_fill


def dense_qkv(wl, cache, scales, b, j=0):
    """q rows of (b, j) for all heads and the dense dequantized K, V per kv head."""
    n = int(wl.seq_lens[b]) - wl.q_len + j + 1
    q = oracle.bf16_to_f64(wl.q[b * wl.q_len + j])
    Ks = [oracle.gather_dequant(cache, scales, wl.mode, wl.block_tables[b], n, 0, h)
          for h in range(wl.num_kv_heads)]
    Vs = [oracle.gather_dequant(cache, scales, wl.mode, wl.block_tables[b], n, 1, h)
          for h in range(wl.num_kv_heads)]
    return q, Ks, Vs, n


def run(wl, cache, scales):
    return oracle.paged_decode_attn(wl.q, cache, scales, wl.mode, wl.block_tables, wl.seq_lens,
                                    wl.q_len, wl.sm_scale)


@pytest.mark.parametrize("mode", [W.MODE_INT8, W.MODE_FP8, W.MODE_FP8_TENSOR, W.MODE_INT4,
                                  W.MODE_INT4_GROUP])
def test_tiny_config_equals_dense_brute_force(mode):
    wl = W.tiny(mode)
    cache, scales = oracle_fill(wl)
    out = run(wl, cache, scales)
    assert out.shape == (2, 4, 64)
    G = wl.group
    for b in range(wl.batch):
        q, Ks, Vs, n = dense_qkv(wl, cache, scales, b)
        assert n == wl.seq_lens[b]
        for h in range(wl.num_kv_heads):
            want, w = brute.dense_attention(q[h * G:(h + 1) * G], Ks[h], Vs[h], wl.sm_scale)
            assert np.allclose(out[b, h * G:(h + 1) * G], want, rtol=0, atol=1e-13)
    # and the dequantized K the attention saw is the quantization of the workload's K
    k, v = wl.kv_rows(1, 0, 100)
    K = oracle.gather_dequant(cache, scales, mode, wl.block_tables[1], 100, 0, 1)
    x = oracle.bf16_to_f64(k[:, 1])
    rel = np.abs(K - x).max() / np.abs(x).max()
    assert rel < {W.MODE_INT8: 0.005, W.MODE_INT4: 0.08, W.MODE_INT4_GROUP: 0.08}.get(mode, 0.07)


def test_unquantized_mode_is_attention_over_the_original_rows():
    """Mode 2 stores the bf16 rows as they are, so the checker's output must be the dense
    attention over the workload's own K and V, gathered here without the checker: this pins
    its slot indexing, table walk and attention loops with no quantization in between."""
    wl = W.custom("plain", W.MODE_BF16, [37, 100, 5], 2, 4, 2, 64, 16, seed=12)
    cache, scales = oracle_fill(wl)
    assert cache.dtype == np.uint16 and scales.size == 0
    out = run(wl, cache, scales)
    G = wl.group
    for b in range(wl.batch):
        L = int(wl.seq_lens[b])
        k, v = wl.kv_rows(b, 0, L)
        for j in range(wl.q_len):
            n = L - wl.q_len + j + 1
            q = oracle.bf16_to_f64(wl.q[b * wl.q_len + j])
            for h in range(wl.num_kv_heads):
                want, _ = brute.dense_attention(q[h * G:(h + 1) * G],
                                                oracle.bf16_to_f64(k[:n, h]),
                                                oracle.bf16_to_f64(v[:n, h]), wl.sm_scale)
                assert np.allclose(out[b * wl.q_len + j, h * G:(h + 1) * G], want, rtol=0, atol=1e-13)
    # the stored bits are the rows' bits, at the slots the table names
    k, v = wl.kv_rows(1, 0, 100)
    for p in (0, 15, 16, 99):
        blk, off = wl.block_tables[1][p // 16], p % 16
        assert np.array_equal(cache[blk, 0, :, off], k[p]) and np.array_equal(cache[blk, 1, :, off], v[p])
    # and quantized attention stays near it (one K channel of the 128 is 20x larger than the
    # rest, which costs int8 per token-head a few percent)
    wq = W.custom("plain", W.MODE_INT8, [37, 100, 5], 2, 4, 2, 64, 16, seed=12)
    assert np.array_equal(wq.q, wl.q)
    cq, sq = oracle_fill(wq)
    assert np.abs(run(wq, cq, sq) - out).max() < 0.10 * np.abs(out).max()


def test_weights_are_a_probability_vector():
    wl = W.tiny()
    cache, scales = oracle_fill(wl)
    for b in range(2):
        for hq in range(4):
            w = oracle.attn_weights(wl.q, cache, scales, wl.mode, wl.block_tables[b],
                                    int(wl.seq_lens[b]), 1, 0, hq, b, wl.sm_scale)
            assert w.shape == (wl.seq_lens[b],)
            assert np.all(w >= 0) and abs(w.sum() - 1.0) < 1e-14


def small_wl(mode, seq_lens, q_len=1, Hq=4, Hkv=2, D=64, bs=16, seed=77):
    return W.custom("small", mode, seq_lens, q_len, Hq, Hkv, D, bs, seed, outliers=False)


@pytest.mark.parametrize("mode", [W.MODE_INT8, W.MODE_FP8])
def test_identical_keys_give_the_mean_of_v(mode):
    """Closed form: if every stored key of a head is the same vector, the weights are uniform
    and the output is the arithmetic mean of the dequantized V rows."""
    wl = small_wl(mode, [45, 16, 1])
    cache, scales = oracle.alloc_cache(mode, wl.num_blocks, 16, 2, 64)
    for b in range(wl.batch):
        L = int(wl.seq_lens[b])
        k, v = wl.kv_rows(b, 0, L)
        k[:] = k[0:1]                       # same key row at every position
        oracle.kv_quant_write(k, v, wl.slots(b, 0, L), cache, scales, mode)
    out = run(wl, cache, scales)
    for b in range(wl.batch):
        L = int(wl.seq_lens[b])
        for hq in range(4):
            V = oracle.gather_dequant(cache, scales, mode, wl.block_tables[b], L, 1, hq // 2)
            assert np.allclose(out[b, hq], V.mean(axis=0), rtol=0, atol=1e-14)


def test_single_position_returns_that_v_row():
    wl = small_wl(W.MODE_INT8, [1, 1])
    cache, scales = oracle_fill(wl)
    out = run(wl, cache, scales)
    for b in range(2):
        for hq in range(4):
            V = oracle.gather_dequant(cache, scales, 0, wl.block_tables[b], 1, 1, hq // 2)
            assert np.array_equal(out[b, hq], V[0])


def test_one_dominant_key_selects_its_v_row():
    wl = small_wl(W.MODE_INT8, [60])
    L = 60
    k, v = wl.kv_rows(0, 0, L)
    qf = W.bf16_bits_to_f32(wl.q[0])                       # [Hq, D]
    # position 41 of kv head 0 gets key = 40 * q of q head 1 (logit = 5 * |q|^2 >> the rest)
    k[41, 0] = W.to_bf16_bits(qf[1] * 40)
    cache, scales = oracle.alloc_cache(0, wl.num_blocks, 16, 2, 64)
    oracle.kv_quant_write(k, v, wl.slots(0, 0, L), cache, scales, 0)
    out = run(wl, cache, scales)
    V = oracle.gather_dequant(cache, scales, 0, wl.block_tables[0], L, 1, 0)
    assert np.allclose(out[0, 1], V[41], rtol=0, atol=1e-9)
    assert not np.allclose(out[0, 0], V[41], atol=1e-3)     # other q head of the group: no


def test_output_is_a_convex_combination_and_group_rows_agree():
    wl = small_wl(W.MODE_FP8, [70, 33], Hq=8, Hkv=2)
    wl.q[:, 1] = wl.q[:, 0]            # q heads 0 and 1 (same kv head) get the same query
    wl.q[:, 4] = wl.q[:, 0]            # q head 4 (other kv head) as well
    cache, scales = oracle_fill(wl)
    out = run(wl, cache, scales)
    for b in range(2):
        assert np.array_equal(out[b, 0], out[b, 1])
        assert not np.allclose(out[b, 0], out[b, 4])
        for hq in range(8):
            V = oracle.gather_dequant(cache, scales, 1, wl.block_tables[b], int(wl.seq_lens[b]), 1,
                                      hq // 4)
            assert np.all(out[b, hq] <= V.max(axis=0) + 1e-15)
            assert np.all(out[b, hq] >= V.min(axis=0) - 1e-15)


def test_gqa_head_mapping_is_contiguous_groups():
    """q head hq reads kv head hq // G: zero every kv head but one and see which q heads move."""
    wl = small_wl(W.MODE_INT8, [40], Hq=8, Hkv=4)
    L = 40
    k, v = wl.kv_rows(0, 0, L)
    v[:, [0, 1, 3]] = 0                 # only kv head 2 has non-zero V
    cache, scales = oracle.alloc_cache(0, wl.num_blocks, 16, 4, 64)
    oracle.kv_quant_write(k, v, wl.slots(0, 0, L), cache, scales, 0)
    out = run(wl, cache, scales)
    moved = [bool(np.abs(out[0, hq]).max() > 0) for hq in range(8)]
    assert moved == [False, False, False, False, True, True, False, False]


@pytest.mark.parametrize("mode", [W.MODE_INT8, W.MODE_FP8])
def test_causal_multi_token_equals_single_token_calls(mode):
    """q_len = 4: query j sees positions 0 .. L - 4 + j.  Equals four q_len = 1 calls with
    seq_lens L - 3 .. L on the same cache."""
    wl = small_wl(mode, [53, 20, 4], q_len=4, Hq=4, Hkv=2)
    cache, scales = oracle_fill(wl)
    out = run(wl, cache, scales).reshape(wl.batch, 4, 4, 64)
    for j in range(4):
        qj = np.ascontiguousarray(wl.q.reshape(wl.batch, 4, 4, 64)[:, j])
        lens = (wl.seq_lens - 4 + j + 1).astype(np.int32)
        single = oracle.paged_decode_attn(qj, cache, scales, mode, wl.block_tables, lens, 1,
                                          wl.sm_scale)
        assert np.array_equal(out[:, j], single)
    # and against the dense brute force with an explicit causal length
    q, Ks, Vs, n = dense_qkv(wl, cache, scales, 0, j=1)
    assert n == 53 - 4 + 2
    want, _ = brute.dense_attention(q[0:2], Ks[0], Vs[0], wl.sm_scale)
    assert np.allclose(out[0, 1, 0:2], want, rtol=0, atol=1e-13)


def test_permuting_physical_blocks_changes_nothing():
    wl = small_wl(W.MODE_INT8, [90, 31])
    cache, scales = oracle_fill(wl)
    out = run(wl, cache, scales)
    rng = np.random.default_rng(3)
    perm = rng.permutation(wl.num_blocks)          # new id of old block i is perm[i]
    cache2, scales2 = np.empty_like(cache), np.empty_like(scales)
    cache2[perm], scales2[perm] = cache, scales
    tables2 = np.where(wl.block_tables >= 0, perm[np.maximum(wl.block_tables, 0)], -1).astype(np.int32)
    out2 = oracle.paged_decode_attn(wl.q, cache2, scales2, wl.mode, tables2, wl.seq_lens, 1,
                                    wl.sm_scale)
    assert np.array_equal(out, out2)


def test_garbage_after_the_last_position_is_never_read():
    wl = small_wl(W.MODE_FP8, [37])
    cache, scales = oracle_fill(wl)
    out = run(wl, cache, scales)
    blk = wl.block_tables[0, 2]
    cache[blk, :, :, 37 - 32:] = 0x7F      # NaN codes in the tail of the last block
    out2 = run(wl, cache, scales)
    assert np.array_equal(out, out2)


def test_split_and_lse_merge_equals_unsplit():
    """The merge rule a split-K evaluation uses, checked in fp64 against the unsplit result."""
    wl = small_wl(W.MODE_INT8, [100])
    cache, scales = oracle_fill(wl)
    out = run(wl, cache, scales)
    q, Ks, Vs, n = dense_qkv(wl, cache, scales, 0)
    for cuts in ([0, 64, 100], [0, 1, 17, 99, 100], [0, 100]):
        parts = [brute.chunk_partial(q[0:2], Ks[0][a:b], Vs[0][a:b], wl.sm_scale)
                 for a, b in zip(cuts[:-1], cuts[1:])]
        assert np.allclose(brute.lse_merge(parts), out[0, 0:2], rtol=0, atol=1e-14)


def test_scaling_q_to_zero_gives_uniform_weights():
    wl = small_wl(W.MODE_INT8, [25])
    wl.q[:] = 0
    cache, scales = oracle_fill(wl)
    out = run(wl, cache, scales)
    V = oracle.gather_dequant(cache, scales, 0, wl.block_tables[0], 25, 1, 1)
    assert np.allclose(out[0, 3], V.mean(axis=0), rtol=0, atol=1e-15)


def test_transposed_operand_would_fail():
    """z_p must be q . K[p] over channels: a key equal to q at one position, orthogonal noise
    elsewhere, must put the weight on that position (a K/V or row/column mix-up would not)."""
    wl = small_wl(W.MODE_INT8, [16], Hq=2, Hkv=2)
    k, v = wl.kv_rows(0, 0, 16)
    k[:] = 0
    e = np.zeros(64, dtype=np.float32)
    e[9] = 30.0
    k[5, 0] = W.to_bf16_bits(e)
    wl.q[0, 0] = W.to_bf16_bits(e)
    cache, scales = oracle.alloc_cache(0, wl.num_blocks, 16, 2, 64)
    oracle.kv_quant_write(k, v, wl.slots(0, 0, 16), cache, scales, 0)
    w = oracle.attn_weights(wl.q, cache, scales, 0, wl.block_tables[0], 16, 1, 0, 0, 0, wl.sm_scale)
    assert w.argmax() == 5 and w[5] > 0.999999
    # closed form: logits are 900/8 at p = 5 and 0 elsewhere
    want = np.exp(112.5) / (np.exp(112.5) + 15)
    assert abs(w[5] - want) < 1e-12


def test_workload_generators_are_reproducible_and_shaped():
    a, b = W.llama8b(batch=4, lo=100, hi=300), W.llama8b(batch=4, lo=100, hi=300)
    assert np.array_equal(a.seq_lens, b.seq_lens) and np.array_equal(a.block_tables, b.block_tables)
    k1, v1 = a.kv_rows(2, 10, 300 if a.seq_lens[2] >= 300 else int(a.seq_lens[2]))
    k2, _ = b.kv_rows(2, 0, int(a.seq_lens[2]))
    assert np.array_equal(k1, k2[10:10 + k1.shape[0]])
    used = a.block_tables[a.block_tables >= 0]
    assert len(np.unique(used)) == len(used) and used.max() < a.num_blocks
    assert a.num_blocks == 2 * len(used)
    assert len(a.outlier_channels) == 10
    kf = W.bf16_bits_to_f32(k2).reshape(-1, 8 * 128)
    ratio = kf[:, a.outlier_channels].std() / np.delete(kf, a.outlier_channels, axis=1).std()
    assert 15 < ratio < 25
    p = W.verify_prefix(batch=3, lo=1100, hi=1300)
    assert np.array_equal(p.block_tables[0, :64], p.block_tables[2, :64])
    ka, _ = p.kv_rows(0, 1000, 1030)
    kb, _ = p.kv_rows(2, 1000, 1030)
    assert np.array_equal(ka[:24], kb[:24]) and not np.array_equal(ka[24:], kb[24:])
    assert p.unique_tokens() == int(p.seq_lens.sum()) - 2 * 1024
    t = W.tiny()
    assert t.algorithmic_bytes()["kv"] == 137 * 2 * 2 * (64 + 4)
