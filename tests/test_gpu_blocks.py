"""GPU parity, block moves between the pool and a packed staging area (device memory and
pinned host memory): bytes and scales equal the CPU checker's index copies bit for bit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_2605_29639_amd import workloads as W
from helpers import gpu_desc, oracle_fill, upload_oracle_cache


def canon(t, desc):
    from paper_2605_29639_amd import kvq
    a = kvq.cache_to_canonical(t, desc).cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.int16 else a


@pytest.mark.parametrize("host", [False, True], ids=["device", "pinned_host"])
@pytest.mark.parametrize("mode", [W.MODE_INT8, W.MODE_FP8, W.MODE_BF16, W.MODE_FP8_TENSOR,
                                  W.MODE_INT4, W.MODE_INT4_GROUP])
@pytest.mark.parametrize("bs,D,H", [(16, 128, 8), (64, 64, 3)])
def test_export_then_import_elsewhere(mode, host, bs, D, H):
    import torch
    from paper_2605_29639_amd import kvq
    if mode in (W.MODE_INT4, W.MODE_INT4_GROUP) and D != 128:
        pytest.skip("int4 takes head_dim 128 only")
    wl = W.custom("blocks", mode, [300, 77, 150], 1, H, H, D, bs, seed=5 + bs + mode)
    oc, osc = oracle_fill(wl)
    cache, scales, desc = upload_oracle_cache(wl, oc, osc)
    rng = np.random.default_rng(3)
    ids = rng.permutation(wl.num_blocks)[:max(1, wl.num_blocks // 2)].astype(np.int32)
    n = len(ids)
    cbytes, sfloats = kvq.packed_sizes(desc, n)
    where = dict(pin_memory=True) if host else dict(device="cuda")
    pc = torch.full((cbytes,), 0xEE, dtype=torch.uint8, **where)
    ps = torch.full((sfloats,), -1.0, dtype=torch.float32, **where)
    d_ids = torch.from_numpy(ids).cuda()
    kvq.blocks_export(cache, scales, desc, d_ids, pc, ps)
    torch.cuda.synchronize()
    want_c, want_s = oracle.blocks_export(oc, osc, mode, ids)
    pdesc = kvq.make_desc(mode, n, bs, H, D)          # the packed area is a pool of n blocks
    assert np.array_equal(canon(pc.cuda(), pdesc), want_c)
    if mode in (W.MODE_INT8, W.MODE_FP8, W.MODE_INT4, W.MODE_INT4_GROUP):
        assert np.array_equal(ps.cpu().numpy().view(np.uint32).reshape(want_s.shape),
                              want_s.view(np.uint32))
    # import into a second pool at other places
    pool_c, pool_s = oracle.alloc_cache(mode, wl.num_blocks, bs, H, D)
    pool_c[:] = 0x11
    pool_s[...] = 7.0
    cache2, scales2, _ = upload_oracle_cache(wl, pool_c, pool_s)
    dst = rng.permutation(wl.num_blocks)[:n].astype(np.int32)
    kvq.blocks_import(pc, ps, desc, torch.from_numpy(dst).cuda(), cache2, scales2)
    torch.cuda.synchronize()
    oracle.blocks_import(want_c, want_s, mode, dst, pool_c, pool_s)
    assert np.array_equal(canon(cache2, desc), pool_c)
    assert np.array_equal(scales2.cpu().numpy().view(np.uint32), pool_s.view(np.uint32))


def test_no_blocks_is_a_no_op():
    import torch
    from paper_2605_29639_amd import kvq
    desc = kvq.make_desc(0, 4, 16, 2, 64)
    cache, scales = kvq.alloc_cache(desc)
    empty = torch.empty(0, dtype=torch.int32, device="cuda")
    kvq.blocks_export(cache, scales, desc, empty, torch.empty(0, dtype=torch.uint8, device="cuda"),
                      torch.empty(0, dtype=torch.float32, device="cuda"))
    torch.cuda.synchronize()
