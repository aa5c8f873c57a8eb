"""Pins for the CPU checker's quantization half (CPU only).

Nothing here compares the checker with itself: every expected value comes from a
hand-computed fixture, exact rational arithmetic, a closed form of the format, an
invariant of the method, or torch's own CPU float8 cast.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2605_29639_amd import workloads as W


def f32_bits_of(x):
    return W.to_bf16_bits(np.asarray(x, dtype=np.float32))


def bf16_exact(x):
    """bf16 bit pattern of a value that must be exactly representable."""
    bits = f32_bits_of([x])
    assert float(W.bf16_bits_to_f32(bits)[0]) == float(x), x
    return bits[0]


def read_table(path):
    rows = []
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                rows.append(line)
    return rows


def rne_fraction(fr):
    """Round a Fraction to the nearest integer, ties to even."""
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


def nearest_f32(fr):
    """Correctly rounded fp32 (ties to even) of a positive Fraction, by exact comparison."""
    cand = np.float32(float(fr))  # double rounding could be off by one ulp: check neighbours
    best = None
    for c in (np.nextafter(cand, np.float32(0)), cand, np.nextafter(cand, np.float32(np.inf))):
        err = abs(Fraction(float(c)) - fr)
        key = (err, int(np.float32(c).view(np.uint32)) & 1)
        if best is None or key < best[0]:
            best = (key, np.float32(c))
    return best[1]


# ----------------------------------------------------------------------------- int8

def write_rows_int8(k_rows, v_rows=None):
    """Write T rows (float values exact in bf16) for 1 head into a fresh pool; returns
    (codes int8 [T, D], scales [T]) for K."""
    k_rows = np.asarray(k_rows, dtype=np.float32)
    T, D = k_rows.shape
    kb = f32_bits_of(k_rows).reshape(T, 1, D)
    vb = kb.copy() if v_rows is None else f32_bits_of(np.asarray(v_rows, np.float32)).reshape(T, 1, D)
    bs = 16
    nblk = (T + bs - 1) // bs
    cache, scales = oracle.alloc_cache(oracle.MODE_INT8, nblk, bs, 1, D)
    oracle.kv_quant_write(kb, vb, np.arange(T, dtype=np.int64), cache, scales, oracle.MODE_INT8)
    codes = cache[:, 0, 0].reshape(nblk * bs, D)[:T].view(np.int8)
    sc = scales[:, 0, 0].reshape(nblk * bs)[:T]
    return codes, sc, cache, scales


def test_int8_hand_computed_ties(golden_dir):
    rows = read_table(os.path.join(golden_dir, "int8_ties.txt"))
    xs = [float(r[0]) for r in rows]
    want = [int(r[1]) for r in rows]
    D = 64
    row = np.zeros(D, dtype=np.float32)
    row[:len(xs)] = xs
    for x in xs:
        bf16_exact(x)
    codes, sc, _, _ = write_rows_int8(row[None, :])
    assert sc[0] == np.float32(1.0)
    assert codes[0, :len(xs)].tolist() == want
    assert not codes[0, len(xs):].any()


def test_int8_codes_equal_exact_rational_rounding():
    rng = np.random.default_rng(7)
    T, D = 1500, 128
    x = rng.standard_normal((T, D), dtype=np.float32)
    x[:, 5] *= 20.0
    bits = f32_bits_of(x)
    xv = W.bf16_bits_to_f32(bits)
    codes, sc, _, _ = write_rows_int8(xv)
    for t in range(T):
        m = Fraction(float(np.abs(xv[t]).max()))
        assert sc[t] == nearest_f32(m / 127), t
        s = Fraction(float(sc[t]))
        want = [max(-127, min(127, rne_fraction(Fraction(float(v)) / s))) for v in xv[t]]
        assert codes[t].tolist() == want, t


def test_int8_ties_with_a_scale_other_than_one():
    """absmax 254 gives s = 2.0 exactly: 5 -> 2.5 -> 2, 7 -> 3.5 -> 4, 253 -> 126.5 -> 126."""
    row = np.zeros(64, dtype=np.float32)
    row[:6] = [254.0, 5.0, 7.0, 253.0, -5.0, -7.0]
    codes, sc, _, _ = write_rows_int8(row[None, :])
    assert sc[0] == np.float32(2.0)
    assert codes[0, :6].tolist() == [127, 2, 4, 126, -2, -4]


def test_int8_scale_is_correctly_rounded_for_every_bf16_absmax():
    # every positive normal bf16 value as a row's absmax
    hi = np.arange(0x0080, 0x7F80, dtype=np.uint32)
    m = (hi << np.uint32(16)).view(np.float32)
    step = 37  # 32512 values; exact rational check on a stride, all values via the bound below
    for v in m[::step]:
        assert oracle.scale(float(v), 127.0) == nearest_f32(Fraction(float(v)) / 127)
        assert oracle.scale(float(v), 448.0) == nearest_f32(Fraction(float(v)) / 448)
    # all of them: |s - m/127| <= half an ulp of s, evaluated with exact integers
    s = np.array([oracle.scale(float(v), 127.0) for v in m], dtype=np.float32)
    ulp = np.spacing(s).astype(np.float64)
    err = np.abs(s.astype(np.float64) * 127.0 - m.astype(np.float64)) / 127.0  # exact: 24b*7b
    assert np.all(err <= ulp / 2 * (1 + 1e-12))


def test_int8_round_trip_bound_and_saturation():
    rng = np.random.default_rng(11)
    x = rng.standard_normal((400, 128), dtype=np.float32) * rng.uniform(1e-3, 50, (400, 1)).astype(np.float32)
    xv = W.bf16_bits_to_f32(f32_bits_of(x)).astype(np.float64)
    codes, sc, _, _ = write_rows_int8(xv)
    s = sc.astype(np.float64)[:, None]
    err = np.abs(xv - codes.astype(np.float64) * s)
    assert np.all(err <= s / 2 * (1 + 1e-12))
    assert err.max() > 0.49 * s.min()            # the bound is reached, not a loose one
    assert np.all(np.abs(codes.astype(np.int32)).max(axis=1) == 127)   # absmax hits +-127
    assert codes.min() >= -127                                           # -128 never produced


def test_int8_power_of_two_scaling_and_sign_symmetry():
    rng = np.random.default_rng(12)
    x = W.bf16_bits_to_f32(f32_bits_of(rng.standard_normal((50, 64), dtype=np.float32)))
    c1, s1, _, _ = write_rows_int8(x)
    c2, s2, _, _ = write_rows_int8(x * np.float32(2.0 ** -9))
    c3, s3, _, _ = write_rows_int8(-x)
    assert np.array_equal(c1, c2) and np.array_equal(s1 * np.float32(2.0 ** -9), s2)
    assert np.array_equal(c3.astype(np.int32), -c1.astype(np.int32)) and np.array_equal(s1, s3)


def test_int8_zero_row_and_skipped_token():
    D = 64
    k = np.zeros((3, 1, D), dtype=np.uint16)
    k[1, 0, :] = bf16_exact(1.0)
    k[2, 0, 3] = 0x8000  # -0.0 in an otherwise zero row
    cache, scales = oracle.alloc_cache(oracle.MODE_INT8, 1, 16, 1, D)
    cache[:] = 0xAB
    scales[:] = 9.0
    oracle.kv_quant_write(k, k.copy(), np.array([0, -1, 2], dtype=np.int64), cache, scales, 0)
    assert scales[0, 0, 0, 0] == 0.0 and not cache[0, 0, 0, 0].any()       # zero row
    assert scales[0, 0, 0, 2] == 0.0 and not cache[0, 0, 0, 2].any()       # -0.0 row
    assert scales[0, 0, 0, 1] == 9.0 and np.all(cache[0, 0, 0, 1] == 0xAB)  # skipped token
    assert np.all(cache[0, :, 0, 3:] == 0xAB)                               # untouched slots


# ----------------------------------------------------------------------------- fp8 format

def test_fp8_decode_landmarks(golden_dir):
    for code, val in read_table(os.path.join(golden_dir, "e4m3fn_landmarks.txt")):
        got = oracle.fp8_decode(np.uint8(int(code, 16)))
        if val == "nan":
            assert np.isnan(got)
        else:
            assert got == float(val) and np.signbit(got) == val.startswith("-"), code


def test_fp8_decode_all_codes_against_torch_cast():
    codes = np.arange(256, dtype=np.uint8)
    got = oracle.fp8_decode(codes)
    ref = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    nan = np.isnan(ref)
    assert nan.sum() == 2 and np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))


def test_fp8_encode_round_trips_every_finite_code():
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    assert codes.size == 254
    assert np.array_equal(oracle.fp8_encode(oracle.fp8_decode(codes)), codes)


def test_fp8_encode_midpoints_go_to_even_and_neighbours_to_nearer():
    mags = oracle.fp8_decode(np.arange(0x7F, dtype=np.uint8))  # ascending magnitudes
    for c in range(0x7E):
        lo, hi = mags[c], mags[c + 1]
        mid = (lo + hi) / 2  # exact in fp64
        even = c if c % 2 == 0 else c + 1
        assert oracle.fp8_encode(mid) == even
        assert oracle.fp8_encode(-mid) == (0x80 | even)
        assert oracle.fp8_encode(np.nextafter(mid, 0.0)) == c
        assert oracle.fp8_encode(np.nextafter(mid, np.inf)) == c + 1
    assert oracle.fp8_encode(2.0 ** -10) == 0x00          # tie between 0 and 2^-9 -> 0
    assert oracle.fp8_encode(-(2.0 ** -10)) == 0x80       # sign kept on a zero result
    assert oracle.fp8_encode(-1e-30) == 0x80


def test_fp8_encode_saturates_and_never_makes_nan():
    for y in (448.0, 449.0, 463.9, 464.0, 480.0, 1e6, 1e300):
        assert oracle.fp8_encode(y) == 0x7E and oracle.fp8_encode(-y) == 0xFE


def test_fp8_encode_matches_torch_cast_on_exact_fp32_inputs():
    rng = np.random.default_rng(5)
    x = rng.standard_normal(20000).astype(np.float32) * rng.choice(
        np.array([1e-3, 1e-2, 0.1, 1, 10, 100], dtype=np.float32), 20000)
    x = x[np.abs(x) <= 448]
    want = torch.from_numpy(x.copy()).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(oracle.fp8_encode(x.astype(np.float64)), want)


def test_fp8_round_trip_error_bound():
    rng = np.random.default_rng(6)
    y = np.concatenate([rng.uniform(-448, 448, 5000), rng.uniform(-1, 1, 5000) * 2.0 ** -5])
    back = oracle.fp8_decode(oracle.fp8_encode(y))
    big = np.abs(y) >= 2.0 ** -6
    assert np.all(np.abs(back[big] - y[big]) <= np.abs(y[big]) * 2.0 ** -4)
    assert np.all(np.abs(back[~big] - y[~big]) <= 2.0 ** -10)


# ----------------------------------------------------------------------------- fp8 write

def fp8_pool(nblk=4, bs=16, H=1, D=64):
    return oracle.alloc_cache(oracle.MODE_FP8, nblk, bs, H, D)


def test_fp8_block_with_absmax_448_equals_torch_cast():
    """A block whose absmax is 448 has scale exactly 1, so its codes are the plain e4m3
    cast of the values: a library routine (torch's CPU cast) gives the expected bytes."""
    rng = np.random.default_rng(21)
    bs, D = 16, 64
    x = rng.standard_normal((bs, 1, D), dtype=np.float32) * 60
    x = np.clip(W.bf16_bits_to_f32(f32_bits_of(x)), -440, 440)
    x = W.bf16_bits_to_f32(f32_bits_of(x))
    x[3, 0, 7] = 448.0
    kb = f32_bits_of(x)
    vb = f32_bits_of(-x)
    cache, scales = fp8_pool()
    oracle.kv_quant_write(kb, vb, np.arange(bs, 2 * bs, dtype=np.int64), cache, scales, 1)
    assert scales[1, 0, 0] == 1.0 and scales[1, 1, 0] == 1.0
    want_k = torch.from_numpy(x.copy()).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    want_v = torch.from_numpy((-x).copy()).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(cache[1, 0, 0], want_k[:, 0])
    assert np.array_equal(cache[1, 1, 0], want_v[:, 0])
    assert not cache[0].any() and not cache[2:].any()


def test_fp8_one_shot_block_codes_equal_exact_rational_rounding():
    rng = np.random.default_rng(22)
    bs, D = 16, 64
    x = W.bf16_bits_to_f32(f32_bits_of(rng.standard_normal((bs, 1, D), dtype=np.float32) * 3))
    cache, scales = fp8_pool()
    oracle.kv_quant_write(f32_bits_of(x), f32_bits_of(x), np.arange(bs, dtype=np.int64), cache,
                          scales, 1)
    m = Fraction(float(np.abs(x).max()))
    assert scales[0, 0, 0] == nearest_f32(m / 448)
    s = Fraction(float(scales[0, 0, 0]))
    mags = [Fraction(float(v)) for v in oracle.fp8_decode(np.arange(0x7F, dtype=np.uint8))]
    for t in range(bs):
        for d in range(D):
            y = Fraction(float(x[t, 0, d])) / s
            a = min(abs(y), Fraction(448))
            errs = [(abs(mg - a), c & 1, c) for c, mg in enumerate(mags)]
            want = min(errs)[2] | (0x80 if x[t, 0, d] < 0 or np.signbit(x[t, 0, d]) else 0)
            assert cache[0, 0, 0, t, d] == want


def test_fp8_append_invariants():
    rng = np.random.default_rng(23)
    bs, D, H = 16, 64, 2
    x = W.bf16_bits_to_f32(f32_bits_of(rng.standard_normal((bs, H, D), dtype=np.float32)))
    x[5] *= 4.0      # token 5 raises the block absmax
    x[9] *= 0.25     # token 9 is small
    x = W.bf16_bits_to_f32(f32_bits_of(x))
    bits = f32_bits_of(x)
    cache, scales = fp8_pool(H=H)
    scales[:] = 123.0    # stale scale: must be ignored by the write at offset 0
    cache[:] = 0x55
    blk = 2
    growths = np.zeros(H, dtype=np.int64)
    for t in range(bs):
        before = cache[blk].copy()
        s_before = scales[blk].copy()
        oracle.kv_quant_write(bits[t:t + 1], bits[t:t + 1],
                              np.array([blk * bs + t], dtype=np.int64), cache, scales, 1)
        # stored scale = fp32(absmax of the live tokens / 448), for every head, K and V
        for h in range(H):
            want = nearest_f32(Fraction(float(np.abs(x[:t + 1, h]).max())) / 448)
            assert scales[blk, 0, h] == want and scales[blk, 1, h] == want
        grew = scales[blk] > s_before
        growths += grew[0] if t > 0 else 0
        for h in range(H):
            if t > 0 and not grew[0, h]:
                # a token that does not raise the absmax changes no earlier byte
                assert np.array_equal(cache[blk, 0, h, :t], before[0, h, :t])
        assert np.all(cache[blk, :, :, t + 1:] == 0x55)   # later slots untouched
    assert np.all(cache[[0, 1, 3]] == 0x55)
    # every stored value went through at most (growths + 1) roundings, each within half an
    # e4m3 step (relative 2^-4 for normals, absolute s * 2^-10 for subnormals)
    deq = oracle.dequant(cache, scales, 1)[blk, 0]
    assert growths.min() >= 1
    for h in range(H):
        s = float(scales[blk, 0, h])
        n = growths[h] + 1
        tol = n * (np.abs(x[:, h]) * 2.0 ** -4 * 1.07 + s * 2.0 ** -10)
        assert np.all(np.abs(deq[h] - x[:, h]) <= tol)


def test_fp8_rescale_is_the_stated_re_encoding():
    """After the scale grows from s0 to s1, an earlier code c must hold
    encode(decode(c) * s0 / s1) evaluated exactly."""
    bs, D = 16, 64
    rng = np.random.default_rng(24)
    x0 = W.bf16_bits_to_f32(f32_bits_of(rng.standard_normal((3, 1, D), dtype=np.float32)))
    x1 = W.bf16_bits_to_f32(f32_bits_of(rng.standard_normal((1, 1, D), dtype=np.float32) * 7))
    cache, scales = fp8_pool()
    oracle.kv_quant_write(f32_bits_of(x0), f32_bits_of(x0), np.arange(3, dtype=np.int64), cache,
                          scales, 1)
    c0, s0 = cache[0, 0, 0, :3].copy(), Fraction(float(scales[0, 0, 0]))
    oracle.kv_quant_write(f32_bits_of(x1), f32_bits_of(x1), np.array([3], dtype=np.int64), cache,
                          scales, 1)
    s1 = Fraction(float(scales[0, 0, 0]))
    assert s1 > s0
    mags = [Fraction(float(v)) for v in oracle.fp8_decode(np.arange(0x7F, dtype=np.uint8))]
    for t in range(3):
        for d in range(D):
            c = int(c0[t, d])
            y = mags[c & 0x7F] * s0 / s1
            want = min((abs(mg - y), k & 1, k) for k, mg in enumerate(mags))[2] | (c & 0x80)
            assert cache[0, 0, 0, t, d] == want


def test_fp8_whole_block_in_one_call_equals_any_split_when_scale_never_grows():
    rng = np.random.default_rng(25)
    bs, D = 16, 64
    x = W.bf16_bits_to_f32(f32_bits_of(rng.standard_normal((bs, 1, D), dtype=np.float32)))
    x[0, 0, 0] = 100.0  # the first token already carries the block absmax
    bits = f32_bits_of(x)
    a_cache, a_scales = fp8_pool()
    oracle.kv_quant_write(bits, bits, np.arange(bs, dtype=np.int64), a_cache, a_scales, 1)
    b_cache, b_scales = fp8_pool()
    for lo, hi in ((0, 5), (5, 6), (6, 16)):
        oracle.kv_quant_write(bits[lo:hi], bits[lo:hi], np.arange(lo, hi, dtype=np.int64), b_cache,
                              b_scales, 1)
    assert np.array_equal(a_cache, b_cache) and np.array_equal(a_scales, b_scales)


def test_fp8_zero_block_and_fresh_block_rule():
    bs, D = 16, 64
    cache, scales = fp8_pool()
    scales[:] = 5.0
    z = np.zeros((2, 1, D), dtype=np.uint16)
    z[1, 0, 0] = 0x8000
    oracle.kv_quant_write(z, z, np.array([0, 1], dtype=np.int64), cache, scales, 1)
    assert scales[0, 0, 0] == 0.0 and not cache[0, :, :, :2].any()
    # appending real data to a block whose scale is 0: no re-encode (nothing to rescale)
    one = np.full((1, 1, D), bf16_exact(448.0), dtype=np.uint16)
    oracle.kv_quant_write(one, one, np.array([2], dtype=np.int64), cache, scales, 1)
    assert scales[0, 0, 0] == 1.0 and np.all(cache[0, 0, 0, 2] == 0x7E)
    assert not cache[0, :, :, :2].any()


# ----------------------------------------------------------------------------- indexing

@pytest.mark.parametrize("mode", [0, 1])
def test_slot_indexing_identity_through_a_permuted_table(mode):
    """Rows whose values spell out (token, head, channel) in small integers, with a planted
    absmax that makes the scale exactly 1, written through a random table and gathered
    back through it."""
    rng = np.random.default_rng(31)
    bs, H, D, T = 16, 2, 64, 53
    nblk = 9
    table = rng.permutation(nblk)[:(T + bs - 1) // bs].astype(np.int32)
    qmax = 127.0 if mode == 0 else 448.0
    t_i, h_i, d_i = np.meshgrid(np.arange(T), np.arange(H), np.arange(D), indexing="ij")
    k = ((t_i * 3 + h_i * 5 + d_i) % 15 + 1).astype(np.float32)   # 1..15: exact in e4m3 and int8
    v = ((t_i * 7 + h_i + d_i * 2) % 15 + 1).astype(np.float32) * -1
    k[:, :, 0] = qmax
    v[:, :, 0] = -qmax
    p = np.arange(T)
    slots = (table[p // bs].astype(np.int64) * bs + p % bs)
    order = rng.permutation(T) if mode == 0 else np.arange(T)  # int8 rows may come in any order
    cache, scales = oracle.alloc_cache(mode, nblk, bs, H, D)
    oracle.kv_quant_write(f32_bits_of(k)[order], f32_bits_of(v)[order], slots[order], cache,
                          scales, mode)
    for h in range(H):
        K = oracle.gather_dequant(cache, scales, mode, table, T, 0, h)
        V = oracle.gather_dequant(cache, scales, mode, table, T, 1, h)
        assert np.array_equal(K, k[:, h].astype(np.float64))
        assert np.array_equal(V, v[:, h].astype(np.float64))
    # the canonical layout itself: element (blk, kv, h, off, d)
    deq = oracle.dequant(cache, scales, mode)
    for t in (0, 17, T - 1):
        assert np.array_equal(deq[slots[t] // bs, 0, :, slots[t] % bs], k[t].astype(np.float64))
        assert np.array_equal(deq[slots[t] // bs, 1, :, slots[t] % bs], v[t].astype(np.float64))


def test_footprint_is_half_of_bf16():
    """Section 7.2.2: an INT8 / FP8 cache is half the size of the BF16 one."""
    for mode, bs, D in ((0, 16, 128), (1, 16, 128), (0, 64, 128)):
        cache, scales = oracle.alloc_cache(mode, 10, bs, 8, D)
        ratio = (cache.nbytes + scales.nbytes) / (10 * 2 * 8 * bs * D * 2)
        assert 0.5 <= ratio <= 0.52


@pytest.mark.parametrize("mode", [W.MODE_INT8, W.MODE_FP8, W.MODE_BF16, W.MODE_FP8_TENSOR, W.MODE_INT4,
                                  W.MODE_INT4_GROUP])
def test_block_export_and_import_move_whole_blocks_and_nothing_else(mode):
    """The tiered cache's block moves are index copies: checked element by element against
    explicit loops, as a round trip, and for leaving every other block alone."""
    rng = np.random.default_rng(17 + mode)
    nblk, bs, H, D = 9, 16, 2, 64
    cache, scales = oracle.alloc_cache(mode, nblk, bs, H, D)
    cache[:] = rng.integers(0, 1 << (8 * cache.itemsize), size=cache.shape, dtype=np.uint32).astype(cache.dtype)
    scales[...] = rng.random(scales.shape, dtype=np.float32)
    per_block_scales = mode in (W.MODE_INT8, W.MODE_FP8, W.MODE_INT4, W.MODE_INT4_GROUP)
    ids = np.array([7, 0, 3], dtype=np.int32)
    pc, ps = oracle.blocks_export(cache, scales, mode, ids)
    assert pc.shape == (3,) + cache.shape[1:]
    for i, blk in enumerate(ids):
        for kv in range(2):
            for h in range(H):
                assert np.array_equal(pc[i, kv, h], cache[blk, kv, h])
                if per_block_scales:
                    assert np.array_equal(ps[i, kv, h], scales[blk, kv, h])
    # import into another pool at other ids: those blocks change, the rest do not
    pool, pscales = oracle.alloc_cache(mode, nblk, bs, H, D)
    pool[:] = 0x5A
    pscales[...] = 9.0
    before, before_s = pool.copy(), pscales.copy()
    dst = np.array([1, 8, 4], dtype=np.int32)
    oracle.blocks_import(pc, ps, mode, dst, pool, pscales)
    for i, blk in enumerate(dst):
        assert np.array_equal(pool[blk], cache[ids[i]])
    others = [b for b in range(nblk) if b not in dst]
    assert np.array_equal(pool[others], before[others])
    if per_block_scales:
        assert np.array_equal(pscales[dst], scales[ids]) and np.array_equal(pscales[others], before_s[others])
    else:
        assert np.array_equal(pscales, before_s)
    # round trip
    back, back_s = oracle.blocks_export(pool, pscales, mode, dst)
    assert np.array_equal(back, pc) and (not per_block_scales or np.array_equal(back_s, ps))


def test_static_per_tensor_fp8_codes():
    """Mode 3: the write only encodes x / s with the caller's two scales.  Pinned by (a) every
    finite code times a power-of-two scale coming back as itself, (b) torch's e4m3 cast of the
    exactly representable quotient for a power-of-two scale, (c) exact rational rounding and
    saturation for a scale that is not a power of two; the scales are never modified and the
    K scale is not used for V."""
    bs, D = 16, 64
    # (a) 254 finite codes = 4 tokens of 64 channels (NaN codes 0x7F / 0xFF left out)
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    vals = oracle.fp8_decode(codes)
    x = np.zeros((bs, 1, D))
    x.reshape(-1)[:codes.size] = vals * 2.0 ** -3
    xb = f32_bits_of(x.astype(np.float32))
    assert np.array_equal(W.bf16_bits_to_f32(xb).astype(np.float64), x)   # bf16-exact inputs
    cache, scales = oracle.alloc_cache(3, 2, bs, 1, D)
    scales[:] = (2.0 ** -3, 2.0 ** 5)
    oracle.kv_quant_write(xb, xb, np.arange(bs, dtype=np.int64), cache, scales, 3)
    assert scales.tolist() == [2.0 ** -3, 2.0 ** 5]
    got = cache[0, 0, 0].reshape(-1)[:codes.size]
    assert np.array_equal(got & 0x7F, codes & 0x7F)
    assert np.array_equal((got >> 7)[vals != 0], (codes >> 7)[vals != 0])
    # V used its own scale: the same inputs over 2^5 are 256 times smaller
    want_v = oracle.fp8_encode(x.reshape(-1)[:codes.size] / 2.0 ** 5)
    assert np.array_equal(cache[0, 1, 0].reshape(-1)[:codes.size], want_v)
    # (b) random bf16 rows, power-of-two scale: x / s is exact in fp32, torch casts it
    rng = np.random.default_rng(40)
    x = W.bf16_bits_to_f32(f32_bits_of(rng.standard_normal((bs, 1, D), dtype=np.float32) * 3))
    s = np.float32(2.0 ** -6)
    scales[:] = (s, s)
    oracle.kv_quant_write(f32_bits_of(x), f32_bits_of(x), np.arange(bs, 2 * bs, dtype=np.int64),
                          cache, scales, 3)
    y = torch.from_numpy(np.clip(x / s, -448, 448)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(cache[1, 0, 0], y[:, 0])
    # (c) a scale that is no power of two; some values saturate
    s = np.float32(0.0123)
    scales[:] = (s, s)
    oracle.kv_quant_write(f32_bits_of(x), f32_bits_of(x), np.arange(bs, dtype=np.int64), cache,
                          scales, 3)
    mags = [Fraction(float(v)) for v in oracle.fp8_decode(np.arange(0x7F, dtype=np.uint8))]
    saturated = 0
    for t in range(bs):
        for d in range(0, D, 3):
            yq = Fraction(float(x[t, 0, d])) / Fraction(float(s))
            saturated += abs(yq) > 448
            a = min(abs(yq), Fraction(448))
            want = min((abs(mg - a), c & 1, c) for c, mg in enumerate(mags))[2]
            want |= 0x80 if np.signbit(x[t, 0, d]) else 0
            assert cache[0, 1, 0, t, d] == want
    assert saturated > 0
    # dequantized values are code * tensor scale
    dq = oracle.dequant(cache, scales, 3)
    assert dq[0, 1, 0, 3, 6] == oracle.fp8_decode(cache[0, 1, 0, 3, 6]) * float(s)
    # a zero scale gives zero codes
    scales[:] = (0.0, s)
    oracle.kv_quant_write(f32_bits_of(x), f32_bits_of(x), np.arange(bs, dtype=np.int64), cache,
                          scales, 3)
    assert not cache[0, 0].any() and cache[0, 1].any()


# ---------------------------------------------------------------------------- int4

def write_rows_int4(k_rows):
    """Write T rows (values exact in bf16) for 1 head into a fresh int4 pool; returns
    (codes int8 [T, D], scales [T], raw cache)."""
    k_rows = np.asarray(k_rows, dtype=np.float32)
    T, D = k_rows.shape
    kb = f32_bits_of(k_rows).reshape(T, 1, D)
    bs = 16
    nblk = (T + bs - 1) // bs
    cache, scales = oracle.alloc_cache(oracle.MODE_INT4, nblk, bs, 1, D)
    oracle.kv_quant_write(kb, kb.copy(), np.arange(T, dtype=np.int64), cache, scales, oracle.MODE_INT4)
    raw = cache[:, 0, 0].reshape(nblk * bs, D // 2)[:T]
    # unpacked here by hand, not with the checker's own helper
    codes = np.empty((T, D), dtype=np.int8)
    codes[:, 0::2] = ((raw & 15).astype(np.int16) ^ 8) - 8
    codes[:, 1::2] = ((raw >> 4).astype(np.int16) ^ 8) - 8
    return codes, scales[:, 0, 0].reshape(nblk * bs)[:T], cache, scales


def test_int4_hand_computed_ties_and_nibble_order(golden_dir):
    rows = read_table(os.path.join(golden_dir, "int4_ties.txt"))
    xs = [float(r[0]) for r in rows]
    want = [int(r[1]) for r in rows]
    D = 64
    row = np.zeros(D, dtype=np.float32)
    row[:len(xs)] = xs
    for x in xs:
        bf16_exact(x)
    codes, sc, cache, _ = write_rows_int4(row[None, :])
    assert sc[0] == np.float32(1.0)
    assert codes[0, :len(xs)].tolist() == want
    assert not codes[0, len(xs):].any()
    # byte 0 holds channel 0 (7 -> 0x7) low and channel 1 (-7 -> 0x9) high; byte 1: 6, 6
    assert cache[0, 0, 0, 0, 0] == 0x97 and cache[0, 0, 0, 0, 1] == 0x66
    assert cache.shape[-1] == D // 2


def test_int4_codes_equal_exact_rational_rounding_and_never_minus_eight():
    rng = np.random.default_rng(71)
    T, D = 600, 128
    x = rng.standard_normal((T, D), dtype=np.float32)
    x[:, 5] *= 3.0
    xv = W.bf16_bits_to_f32(f32_bits_of(x))
    codes, sc, cache, scales = write_rows_int4(xv)
    for t in range(T):
        m = Fraction(float(np.abs(xv[t]).max()))
        assert sc[t] == nearest_f32(m / 7), t
        s = Fraction(float(sc[t]))
        want = [max(-7, min(7, rne_fraction(Fraction(float(v)) / s))) for v in xv[t]]
        assert codes[t].tolist() == want, t
    assert codes.min() == -7 and codes.max() == 7
    assert np.all(np.abs(codes.astype(np.int32)).max(axis=1) == 7)
    # round trip: |x - code * s| <= s / 2, and the checker's own unpack / dequant agree
    s64 = sc.astype(np.float64)[:, None]
    assert np.all(np.abs(xv.astype(np.float64) - codes * s64) <= s64 / 2 * (1 + 1e-12))
    assert np.array_equal(oracle.unpack_int4(cache)[:, 0, 0].reshape(-1, D)[:T], codes)
    dq = oracle.dequant(cache, scales, oracle.MODE_INT4)
    assert np.array_equal(dq[:, 0, 0].reshape(-1, D)[:T], codes * s64)


def test_int4_scale_is_correctly_rounded_and_zero_rows():
    hi = np.arange(0x0080, 0x7F80, 41, dtype=np.uint32)
    for v in (hi << np.uint32(16)).view(np.float32):
        assert oracle.scale(float(v), 7.0) == nearest_f32(Fraction(float(v)) / 7)
    row = np.zeros((2, 64), dtype=np.float32)
    row[1, 3] = -2.0
    codes, sc, cache, _ = write_rows_int4(row)
    assert sc[0] == 0 and not cache[0, 0, 0, 0].any()
    assert sc[1] == np.float32(2.0 / 7) and codes[1, 3] == -7 and np.count_nonzero(codes[1]) == 1


# ---------------------------------------------------------------------------- int4, group scales

def write_rows_int4_group(rows):
    """Write T rows (values exact in bf16) for 1 head into a fresh pool of the group-scaled int4
    format; returns (codes int8 [T, D], scales [T, D / 32], cache, scales array)."""
    rows = np.asarray(rows, dtype=np.float32)
    T, D = rows.shape
    kb = f32_bits_of(rows).reshape(T, 1, D)
    bs = 16
    nblk = (T + bs - 1) // bs
    cache, scales = oracle.alloc_cache(oracle.MODE_INT4_GROUP, nblk, bs, 1, D)
    assert scales.shape == (nblk, 2, 1, bs, D // 32)
    oracle.kv_quant_write(kb, kb.copy(), np.arange(T, dtype=np.int64), cache, scales,
                          oracle.MODE_INT4_GROUP)
    raw = cache[:, 0, 0].reshape(nblk * bs, D // 2)[:T]
    codes = np.empty((T, D), dtype=np.int8)     # unpacked by hand, not with the checker's helper
    codes[:, 0::2] = ((raw & 15).astype(np.int16) ^ 8) - 8
    codes[:, 1::2] = ((raw >> 4).astype(np.int16) ^ 8) - 8
    return codes, scales[:, 0, 0].reshape(nblk * bs, D // 32)[:T], cache, scales


def test_int4_group_scales_hand_computed_ties_per_group(golden_dir):
    """The tie table of the per-token format inside one group (absmax 7: scale 1), next to a
    group whose absmax is 14 (scale 2: 3 -> 1.5 -> 2, 5 -> 2.5 -> 2, -1 -> -0.5 -> 0), an
    all-zero group and a group of small values (scale 2^-10) that keeps its own resolution."""
    rows = read_table(os.path.join(golden_dir, "int4_ties.txt"))
    xs = [float(r[0]) for r in rows]
    want = [int(r[1]) for r in rows]
    assert len(xs) <= 32
    row = np.zeros(128, dtype=np.float32)
    row[32:32 + len(xs)] = xs                       # group 1: the tie table, scale 1
    row[0:6] = [14.0, 3.0, 5.0, -1.0, -14.0, 7.0]   # group 0: scale 2
    row[96:100] = np.array([7.0, -3.5, 1.75, 2.5]) * 2.0 ** -10    # group 3: absmax 7 * 2^-10
    codes, sc, cache, _ = write_rows_int4_group(row[None, :])
    assert sc[0].tolist() == [2.0, 1.0, 0.0, 2.0 ** -10]
    assert codes[0, 32:32 + len(xs)].tolist() == want
    assert codes[0, 0:6].tolist() == [7, 2, 2, 0, -7, 4]        # 7 / 2 = 3.5 -> 4 (even)
    assert not codes[0, 64:96].any()
    assert codes[0, 96:100].tolist() == [7, -4, 2, 2]           # -3.5 -> -4 and 2.5 -> 2 (even)
    # byte 0 holds channel 0 (7 -> 0x7) low and channel 1 (2) high
    assert cache[0, 0, 0, 0, 0] == 0x27 and cache.shape[-1] == 64


def test_int4_group_codes_equal_exact_rational_rounding_group_by_group():
    rng = np.random.default_rng(73)
    T, D = 300, 128
    x = rng.standard_normal((T, D), dtype=np.float32)
    x[:, 5] *= 20.0                                  # an outlier channel in group 0
    xv = W.bf16_bits_to_f32(f32_bits_of(x))
    codes, sc, cache, scales = write_rows_int4_group(xv)
    for t in range(T):
        for g in range(D // 32):
            grp = xv[t, 32 * g:32 * g + 32]
            m = Fraction(float(np.abs(grp).max()))
            assert sc[t, g] == nearest_f32(m / 7), (t, g)
            s = Fraction(float(sc[t, g]))
            want = [max(-7, min(7, rne_fraction(Fraction(float(v)) / s))) for v in grp]
            assert codes[t, 32 * g:32 * g + 32].tolist() == want, (t, g)
    assert codes.min() == -7 and codes.max() == 7
    # every group reaches +-7 and the round trip stays within half of the group's own step
    assert np.all(np.abs(codes.astype(np.int32)).reshape(T, D // 32, 32).max(axis=2) == 7)
    s64 = np.repeat(sc.astype(np.float64), 32, axis=1)
    assert np.all(np.abs(xv.astype(np.float64) - codes * s64) <= s64 / 2 * (1 + 1e-12))
    dq = oracle.dequant(cache, scales, oracle.MODE_INT4_GROUP)
    assert np.array_equal(dq[:, 0, 0].reshape(-1, D)[:T], codes * s64)
    # the outlier costs its own group's resolution only: the other groups' steps stay small
    assert np.median(sc[:, 0]) > 4 * np.median(sc[:, 1:])


def test_int4_group_scales_groups_are_independent_and_reduce_to_the_per_token_format():
    rng = np.random.default_rng(74)
    T, D = 40, 128
    x = W.bf16_bits_to_f32(f32_bits_of(rng.standard_normal((T, D), dtype=np.float32)))
    codes, sc, _, _ = write_rows_int4_group(x)
    y = x.copy()
    y[:, 32:64] *= np.float32(64.0)                  # only group 1 changes
    codes2, sc2, _, _ = write_rows_int4_group(y)
    keep = np.r_[0:32, 64:128]
    assert np.array_equal(codes2[:, keep], codes[:, keep])
    assert np.array_equal(sc2[:, [0, 2, 3]], sc[:, [0, 2, 3]])
    assert np.array_equal(sc2[:, 1], sc[:, 1] * np.float32(64.0))      # a power of two: same codes
    assert np.array_equal(codes2[:, 32:64], codes[:, 32:64])
    # with the same absmax in every group the format is the per-token one
    z = np.clip(x, -3.0, 3.0)
    z[:, [0, 32, 64, 96]] = np.float32(3.5)
    cg, sg, _, _ = write_rows_int4_group(z)
    ct, st, _, _ = write_rows_int4(z)
    assert np.array_equal(cg, ct)
    assert np.array_equal(sg, np.repeat(st[:, None], 4, axis=1))


def test_encoders_clamp_symmetrically_whatever_the_scale():
    """The range is [-127, 127] (int8) and [-7, 7] (int4) also for a quotient beyond it, which a
    row's own scale never produces but a scale taken from elsewhere can: -128 and -8 are never
    codes (configuration 1: "clamped to [-127, 127]")."""
    assert list(oracle.int8_encode(np.array([-1000.0, -127.5, -127.4, 127.5, 1e9]), np.float32(1.0))) \
        == [-127, -127, -127, 127, 127]
    assert list(oracle.int4_encode(np.array([-1000.0, -7.5, -7.4, 7.5, 1e9]), np.float32(1.0))) \
        == [-7, -7, -7, 7, 7]
