"""The C-ABI library: it loads, exports every function the header declares, and rejects bad
arguments on the host before any GPU work (so all of this runs without a GPU)."""
import ctypes as C
import os
import re

import pytest

from paper_2605_29639_amd import kvq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions(name="kvq.h"):
    text = open(os.path.join(ROOT, "include", name)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    text = re.sub(r"^\s*#.*$", "", text, flags=re.M)      # preprocessor lines
    return re.findall(r"\b(\w+)\s*\([^;{}]*\)\s*;", text)


def test_library_loads_and_exports_every_declared_function():
    names = header_functions()
    assert set(names) == set(kvq.EXPORTS) and len(names) == len(kvq.EXPORTS)
    L = kvq.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_measurement_build_exports_the_library_plus_its_switches_and_the_library_none_of_them():
    prof = header_functions("kvq_prof.h")
    assert set(prof) == set(kvq.PROF_EXPORTS) and len(prof) == len(kvq.PROF_EXPORTS)
    P = kvq.prof_lib()
    for n in list(kvq.EXPORTS) + prof:
        assert getattr(P, n) is not None
    L = C.CDLL(kvq.LIB_PATH)
    for n in prof:
        assert not hasattr(L, n), "%s must not be exported by the library proper" % n


def test_strerror_is_static_text_for_any_code():
    for code in (0, -1, -2, -3, -4, -5, -6, -99, 7):
        assert isinstance(kvq.strerror(code), str) and kvq.strerror(code)
    assert kvq.strerror(0) == "ok"


def d(mode=0, nblk=8, bs=16, H=2, D=64):
    return kvq.make_desc(mode, nblk, bs, H, D)


def test_sizes():
    L = kvq.lib()
    assert L.kvq_cache_bytes(C.byref(d())) == 8 * 2 * 2 * 16 * 64
    assert L.kvq_scales_bytes(C.byref(d())) == 8 * 2 * 2 * 16 * 4
    assert L.kvq_scales_bytes(C.byref(d(mode=1))) == 8 * 2 * 2 * 4
    assert L.kvq_cache_bytes(C.byref(d(mode=2))) == 8 * 2 * 2 * 16 * 64 * 2   # unquantized: bf16
    assert L.kvq_scales_bytes(C.byref(d(mode=2))) == 0
    assert L.kvq_cache_bytes(C.byref(d(mode=3))) == 8 * 2 * 2 * 16 * 64       # static fp8 scales:
    assert L.kvq_scales_bytes(C.byref(d(mode=3))) == 8                        # one for K, one for V
    assert L.kvq_cache_bytes(C.byref(d(mode=4, D=128))) == 8 * 2 * 2 * 16 * 64    # int4: two codes a byte
    assert L.kvq_scales_bytes(C.byref(d(mode=4, D=128))) == 8 * 2 * 2 * 16 * 4
    assert L.kvq_cache_bytes(C.byref(d(mode=4, D=64))) == 0                       # head_dim 128 only
    assert L.kvq_cache_bytes(C.byref(d(mode=5, D=128))) == 8 * 2 * 2 * 16 * 64    # int4, group scales:
    assert L.kvq_scales_bytes(C.byref(d(mode=5, D=128))) == 8 * 2 * 2 * 16 * 4 * 4  # four per token-head
    assert L.kvq_cache_bytes(C.byref(d(mode=5, D=64))) == 0
    assert L.kvq_cache_bytes(C.byref(d(D=96))) == 0
    assert L.kvq_cache_bytes(None) == 0


FAKE = C.c_void_p(0x1000)  # never dereferenced: every call below fails validation first


@pytest.mark.parametrize("desc,code", [
    (d(mode=99), kvq.E_BAD_MODE), (d(mode=-1), kvq.E_BAD_MODE),
    (d(bs=8), kvq.E_BAD_SHAPE), (d(bs=48), kvq.E_BAD_SHAPE), (d(bs=512), kvq.E_BAD_SHAPE),
    (d(D=96), kvq.E_BAD_SHAPE), (d(D=256), kvq.E_BAD_SHAPE), (d(H=0), kvq.E_BAD_SHAPE),
    (d(nblk=-1), kvq.E_BAD_SHAPE),
])
def test_write_rejects_bad_descriptors(desc, code):
    L = kvq.lib()
    assert L.kv_quant_write(FAKE, FAKE, FAKE, 4, FAKE, FAKE, C.byref(desc), None) == code


def test_write_argument_checks():
    L = kvq.lib()
    ok = d()
    assert L.kv_quant_write(FAKE, FAKE, FAKE, 4, FAKE, FAKE, None, None) == kvq.E_NULLPTR
    assert L.kv_quant_write(FAKE, FAKE, FAKE, -1, FAKE, FAKE, C.byref(ok), None) == kvq.E_BAD_SHAPE
    assert L.kv_quant_write(None, None, None, 0, None, None, C.byref(ok), None) == kvq.OK
    huge = d(H=4096)                                       # 2^31-1 tokens x 4096 heads: no such grid
    assert L.kv_quant_write(FAKE, FAKE, FAKE, 2 ** 31 - 1, FAKE, FAKE, C.byref(huge), None) == kvq.E_BAD_SHAPE
    odd = C.c_void_p(0x1008)                               # k, v and cache: 16-byte aligned
    assert L.kv_quant_write(odd, FAKE, FAKE, 4, FAKE, FAKE, C.byref(ok), None) == kvq.E_BAD_SHAPE
    assert L.kv_quant_write(FAKE, odd, FAKE, 4, FAKE, FAKE, C.byref(ok), None) == kvq.E_BAD_SHAPE
    assert L.kv_quant_write(FAKE, FAKE, FAKE, 4, odd, FAKE, C.byref(ok), None) == kvq.E_BAD_SHAPE
    for i in range(5):
        args = [FAKE, FAKE, FAKE, 4, FAKE, FAKE]
        args[i if i < 3 else i + 1] = None
        assert L.kv_quant_write(*args, C.byref(ok), None) == kvq.E_NULLPTR


def attn(L, desc, q=FAKE, cache=FAKE, scales=FAKE, tables=FAKE, max_blocks=8, lens=FAKE, batch=2,
         q_len=1, Hq=4, max_len=100, chunk=0, out=FAKE, ws=FAKE, ws_bytes=1 << 30):
    return L.paged_decode_attn(q, cache, scales, C.byref(desc) if desc is not None else None,
                               tables, max_blocks, lens, batch, q_len, Hq, max_len, 0.125, chunk,
                               out, ws, ws_bytes, None)


def test_attn_argument_checks():
    L = kvq.lib()
    ok = d()
    assert attn(L, None) == kvq.E_NULLPTR
    assert attn(L, d(mode=99)) == kvq.E_BAD_MODE
    assert attn(L, ok, Hq=3) == kvq.E_BAD_SHAPE            # 3 % 2 != 0
    assert attn(L, ok, q_len=0) == kvq.E_BAD_SHAPE
    assert attn(L, ok, q_len=1025) == kvq.E_BAD_SHAPE        # above KVQ_MAX_Q_LEN
    assert attn(L, ok, batch=-1) == kvq.E_BAD_SHAPE
    assert attn(L, ok, chunk=100) == kvq.E_BAD_SHAPE       # not a multiple of 64
    assert attn(L, ok, max_blocks=6) == kvq.E_BAD_SHAPE    # 6 * 16 < 100
    assert attn(L, ok, max_len=0) == kvq.E_BAD_SHAPE       # shorter than q_len
    assert attn(L, ok, batch=0) == kvq.OK                  # empty batch: nothing launched
    for name in ("q", "cache", "scales", "tables", "lens", "out"):
        assert attn(L, ok, **{name: None}) == kvq.E_NULLPTR
    for name in ("q", "cache", "out"):                     # read and written in 16-byte pieces
        assert attn(L, ok, **{name: C.c_void_p(0x1008)}) == kvq.E_BAD_SHAPE
    # workspace: one partial slot per (wavefront range, pair) crossing, 16 rows each, and the
    # prefix sums of the sequences' group counts with the shared prefix length behind them
    # (batch + 2 ints, padded to a multiple of 4)
    need = L.paged_decode_attn_workspace_bytes(C.byref(ok), 2, 1, 4, 100, 64)
    flat_max = 2 * 2 * 2                                   # batch * ceil(100/64) * kv heads
    assert need == (flat_max + 2 * 2) * 16 * (64 + 2) * 4 + 4 * 4
    assert attn(L, ok, chunk=64, ws=None) == kvq.E_NULLPTR
    assert attn(L, ok, chunk=64, ws_bytes=need - 1) == kvq.E_WORKSPACE
    assert attn(L, ok, chunk=64, ws=C.c_void_p(0x1004), ws_bytes=need) == kvq.E_BAD_SHAPE
    auto = L.paged_decode_attn_workspace_bytes(C.byref(ok), 2, 1, 4, 100, 0)
    assert auto == need                                    # fewer groups than resident waves
    big = kvq.make_desc(0, 1000, 16, 8, 128)
    assert L.paged_decode_attn_workspace_bytes(C.byref(big), 64, 1, 32, 4096, 0) == \
        (2048 + 64 * 8) * 16 * (128 + 2) * 4 + 68 * 4
    assert L.paged_decode_attn_workspace_bytes(C.byref(big), 1, 1, 33, 100, 0) == 0
    # the group-scaled int4 format: one row tile whatever the row count, one wavefront per SIMD
    g4 = kvq.make_desc(5, 1000, 16, 8, 128)
    assert L.paged_decode_attn_workspace_bytes(C.byref(g4), 128, 4, 64, 16384, 0) == \
        (1024 + 128 * 8 * 2) * 16 * (128 + 2) * 4 + 132 * 4
    # 32 query rows per kv head -> two row tiles -> one resident wavefront per SIMD
    assert L.paged_decode_attn_workspace_bytes(C.byref(big), 128, 4, 64, 16384, 0) == \
        (1024 + 128 * 8) * 32 * (128 + 2) * 4 + 132 * 4
    # with a shared prefix: the prefix kernel's partials behind them, one per pair and piece;
    # 8 kv heads x 32 blocks of 128 stacked rows = 256 walks -> 2 pieces for 512 workgroups
    P = L.paged_decode_attn_prefix_workspace_bytes
    assert P(C.byref(big), 128, 4, 64, 16384, 0, 1024) == \
        (1024 + 128 * 8 * (1 + 2)) * 32 * (128 + 2) * 4 + 132 * 4
    # ... as many pieces as the prefix has 64-token groups at most, and eight at most
    assert P(C.byref(big), 2, 1, 32, 4096, 0, 100) == (1024 + 2 * 8 * (1 + 1)) * 16 * 130 * 4 + 4 * 4
    assert P(C.byref(big), 2, 1, 32, 4096, 0, 4096) == (1024 + 2 * 8 * (1 + 8)) * 16 * 130 * 4 + 4 * 4
    # not used: below 64 tokens, beyond max_seq_len, one sequence, 128 rows and more per kv
    # head, the group-scaled int4 format
    plain = L.paged_decode_attn_workspace_bytes
    for args, desc in (((2, 1, 32, 4096, 0, 63), big), ((2, 1, 32, 4096, 0, 4160), big),
                       ((1, 1, 32, 4096, 0, 1024), big), ((2, 64, 32, 4096, 0, 1024), big),
                       ((2, 1, 32, 4096, 0, 1024), g4)):
        assert P(C.byref(desc), *args) == plain(C.byref(desc), *args[:-1]) > 0, args
    assert P(C.byref(big), 2, 1, 32, 4096, 0, -1) == 0


def test_static_scratch_rejects_what_does_not_fit():
    """Validation on the host: a workspace need above the static buffer's size is an error, not
    a launch (no device pointer below is ever dereferenced)."""
    L = kvq.lib()
    fake = C.c_void_p(0x1000)
    desc = kvq.make_desc(0, 1 << 20, 16, 8, 128)
    batch, q_len, Hq, max_len = 4096, 4, 64, 4096
    assert kvq.workspace_bytes(desc, batch, q_len, Hq, max_len) > kvq.STATIC_WORKSPACE_BYTES
    rc = L.paged_decode_attn_static(fake, fake, fake, C.byref(desc), fake, 256, fake, batch, q_len,
                                    Hq, max_len, 0.1, 0, fake, None)
    assert rc == kvq.E_WORKSPACE
    assert L.paged_decode_attn_static(fake, fake, fake, C.byref(desc), fake, 256, fake, 0, q_len,
                                      Hq, max_len, 0.1, 0, fake, None) == kvq.OK
    assert L.paged_decode_attn_static(None, fake, fake, C.byref(desc), fake, 256, fake, 2, 1,
                                      Hq, max_len, 0.1, 0, fake, None) == kvq.E_NULLPTR


def test_prefix_entry_point_validates_like_the_plain_one():
    L = kvq.lib()
    ok = d()
    args = [FAKE, FAKE, FAKE, C.byref(ok), FAKE, 8, FAKE, 2, 1, 4, 100, 0.125, 0]
    tail = [FAKE, FAKE, 1 << 30, None]
    assert L.paged_decode_attn_prefix(*args, -64, *tail) == kvq.E_BAD_SHAPE
    assert L.paged_decode_attn_prefix(*args[:7], 0, *args[8:], 64, *tail) == kvq.OK   # empty batch
    assert L.paged_decode_attn_prefix(None, *args[1:], 64, *tail) == kvq.E_NULLPTR
    assert L.paged_decode_attn_prefix(*args[:9], 3, *args[10:], 64, *tail) == kvq.E_BAD_SHAPE


def test_repack_argument_checks():
    L = kvq.lib()
    assert L.kvq_cache_to_canonical(None, FAKE, C.byref(d()), None) == kvq.E_NULLPTR
    assert L.kvq_cache_from_canonical(FAKE, FAKE, C.byref(d(D=1)), None) == kvq.E_BAD_SHAPE
    assert L.kvq_cache_to_canonical(None, None, C.byref(d(nblk=0)), None) == kvq.OK


def test_block_move_argument_checks():
    L = kvq.lib()
    ok = d()
    for f in (L.kvq_blocks_export, L.kvq_blocks_import):
        assert f(FAKE, FAKE, None, FAKE, 2, FAKE, FAKE, None) == kvq.E_NULLPTR
        assert f(FAKE, FAKE, C.byref(d(mode=7)), FAKE, 2, FAKE, FAKE, None) == kvq.E_BAD_MODE
        assert f(FAKE, FAKE, C.byref(ok), FAKE, -1, FAKE, FAKE, None) == kvq.E_BAD_SHAPE
        assert f(None, None, C.byref(ok), None, 0, None, None, None) == kvq.OK
        for i in (0, 1, 3, 5, 6):
            args = [FAKE, FAKE, C.byref(ok), FAKE, 2, FAKE, FAKE, None]
            args[i] = None
            assert f(*args) == kvq.E_NULLPTR
        odd = C.c_void_p(0x1004)
        assert f(odd, FAKE, C.byref(ok), FAKE, 2, FAKE, FAKE, None) == kvq.E_BAD_SHAPE
        assert f(FAKE, FAKE, C.byref(ok), FAKE, 2, odd, FAKE, None) == kvq.E_BAD_SHAPE


def test_header_is_plain_c(tmp_path):
    """include/kvq.h is the boundary for C callers: it must compile as C99 and as C++ on its
    own, and a C translation unit that calls every entry point must link against the library."""
    import subprocess
    hdr = os.path.join(ROOT, "include", "kvq.h")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic",
                           "-fsyntax-only", "-x", "c", hdr])
    subprocess.check_call(["g++", "-std=c++11", "-Wall", "-Wextra", "-Werror", "-fsyntax-only",
                           "-x", "c++", hdr])
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic",
                           "-fsyntax-only", "-x", "c", os.path.join(ROOT, "include", "kvq_prof.h")])
    src = tmp_path / "caller.c"
    src.write_text('#include "kvq.h"\n#include <stdio.h>\n'
                   "int main(void) {\n"
                   "  kvq_cache_desc_t d = {KVQ_INT8_TOKEN_HEAD, 8, 16, 2, 64};\n"
                   "  if (kvq_cache_bytes(&d) != 8u * 2 * 2 * 16 * 64) return 1;\n"
                   "  if (kv_quant_write(0, 0, 0, 0, 0, 0, &d, 0) != KVQ_OK) return 2;\n"
                   "  if (paged_decode_attn(0, 0, 0, &d, 0, 8, 0, 0, 1, 4, 100, 0.125f, 0, 0, 0, 0, 0)"
                   " != KVQ_OK) return 3;\n"
                   "  if (kvq_blocks_export(0, 0, &d, 0, 0, 0, 0, 0) != KVQ_OK) return 4;\n"
                   '  puts(kvq_strerror(KVQ_E_WORKSPACE));\n  return 0;\n}\n')
    exe = tmp_path / "caller"
    libdir = os.path.dirname(kvq.LIB_PATH)
    subprocess.check_call(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o",
                           str(exe), "-L", libdir, "-lkvq", "-Wl,-rpath," + libdir])
    out = subprocess.run([str(exe)], stdout=subprocess.PIPE, text=True)
    assert out.returncode == 0 and out.stdout.strip()


def test_binding_rejects_shapes_the_device_would_overrun():
    """The Python binding refuses tensors whose shapes do not fit the descriptor before anything
    reaches the library (CPU tensors are enough: the checks come first)."""
    import torch
    desc = d(nblk=4, bs=16, H=2, D=64)
    cache = torch.zeros(kvq.lib().kvq_cache_bytes(C.byref(desc)), dtype=torch.uint8)
    scales = torch.zeros(kvq.lib().kvq_scales_bytes(C.byref(desc)) // 4, dtype=torch.float32)
    k = torch.zeros((3, 2, 64), dtype=torch.bfloat16)
    slots = torch.zeros(3, dtype=torch.int64)
    with pytest.raises(ValueError):
        kvq.kv_quant_write(k, k[:, :1], slots, cache, scales, desc)          # v: one head short
    with pytest.raises(ValueError):
        kvq.kv_quant_write(k, k, slots[:2], cache, scales, desc)             # a slot short
    with pytest.raises(ValueError):
        kvq.kv_quant_write(k, k, slots, cache[:-16], scales, desc)           # pool too small
    with pytest.raises(ValueError):
        kvq.kv_quant_write(k, k, slots, cache, scales[:-1], desc)
    q = torch.zeros((2, 4, 64), dtype=torch.bfloat16)
    out = torch.zeros((2, 4, 64), dtype=torch.float32)
    bt = torch.zeros((2, 7), dtype=torch.int32)
    sl = torch.ones(2, dtype=torch.int32)
    ws = torch.zeros(1 << 16, dtype=torch.uint8)
    with pytest.raises(ValueError):
        kvq.paged_decode_attn(q[:1], cache, scales, desc, bt, sl, 1, 100, 0.1, out, ws)
    with pytest.raises(ValueError):
        kvq.paged_decode_attn(q, cache, scales, desc, bt, sl, 1, 100, 0.1, out[:, :2], ws)
    with pytest.raises(ValueError):
        kvq.paged_decode_attn(q, cache, scales, desc, bt[:1], sl, 1, 100, 0.1, out, ws)
    with pytest.raises(ValueError):
        kvq.paged_decode_attn(q, cache, scales, desc, bt, sl, 1, 100, 0.1, out, ws[:64])
    with pytest.raises(TypeError):                                           # shapes fit: device check
        kvq.paged_decode_attn(q, cache, scales, desc, bt, sl, 1, 100, 0.1, out, ws)
