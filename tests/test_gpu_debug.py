"""KVQ_DEBUG=1: indices the kernels would follow blindly are checked on the device first and a
violation comes back as KVQ_E_BAD_INDEX: nothing is launched on it, nothing traps or faults,
and the same calls with valid indices still give the checker's results."""
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

import oracle
from paper_2605_29639_amd import workloads as W
from helpers import attn_err, bits_to_bf16_tensor, gpu_desc, oracle_fill


@pytest.fixture
def debug_on():
    old = os.environ.get("KVQ_DEBUG")
    os.environ["KVQ_DEBUG"] = "1"      # read by the library at every call
    yield
    if old is None:
        del os.environ["KVQ_DEBUG"]
    else:
        os.environ["KVQ_DEBUG"] = old


@pytest.mark.parametrize("mode", [W.MODE_INT8, W.MODE_FP8])
def test_bad_indices_are_reported_not_followed(debug_on, mode):
    import torch
    from paper_2605_29639_amd import kvq
    wl = W.custom("debug", mode, [70, 33, 130], 1, 8, 2, 128, 16, seed=11 + mode)
    desc = gpu_desc(wl)
    cache, scales = kvq.alloc_cache(desc)
    before = cache.clone()
    k, v = wl.kv_rows(0, 0, 70)
    kd, vd = bits_to_bf16_tensor(k), bits_to_bf16_tensor(v)
    slots = wl.slots(0, 0, 70)
    bad = slots.copy()
    bad[41] = wl.num_blocks * wl.block_size          # one past the pool's last slot
    with pytest.raises(kvq.KvqError) as e:
        kvq.kv_quant_write(kd, vd, torch.from_numpy(bad).cuda(), cache, scales, desc)
    assert e.value.code == kvq.E_BAD_INDEX
    torch.cuda.synchronize()
    assert torch.equal(cache, before)                # nothing was written

    # the valid calls: same results as without the checks
    for b in range(wl.batch):
        kb, vb = wl.kv_rows(b, 0, int(wl.seq_lens[b]))
        kvq.kv_quant_write(bits_to_bf16_tensor(kb), bits_to_bf16_tensor(vb),
                           torch.from_numpy(wl.slots(b, 0, int(wl.seq_lens[b]))).cuda(), cache,
                           scales, desc)
    oc, osc = oracle_fill(wl)
    want = oracle.paged_decode_attn(wl.q, oc, osc, wl.mode, wl.block_tables, wl.seq_lens, 1, wl.sm_scale)
    q = bits_to_bf16_tensor(wl.q)
    sl = torch.from_numpy(wl.seq_lens).cuda()
    out = torch.zeros((3, 8, 128), dtype=torch.float32, device="cuda")
    ws = kvq.alloc_workspace(desc, 3, 1, 8, wl.max_seq_len)

    def attend(tables, lens):
        kvq.paged_decode_attn(q, cache, scales, desc, tables, lens, 1, wl.max_seq_len, wl.sm_scale,
                              out, ws)
        torch.cuda.synchronize()

    attend(torch.from_numpy(wl.block_tables).cuda(), sl)
    assert attn_err(out.cpu().numpy(), want) <= 2e-3

    for what, tables, lens in (
            ("entry beyond the pool", _with(wl.block_tables, (2, 3), wl.num_blocks), wl.seq_lens),
            ("negative entry in use", _with(wl.block_tables, (0, 4), -1), wl.seq_lens),
            ("length beyond max_seq_len", wl.block_tables, _with(wl.seq_lens, 1, wl.max_seq_len + 1)),
            ("length below q_len", wl.block_tables, _with(wl.seq_lens, 1, 0))):
        out.fill_(7.0)
        with pytest.raises(kvq.KvqError) as e:
            attend(torch.from_numpy(tables).cuda(), torch.from_numpy(lens).cuda())
        assert e.value.code == kvq.E_BAD_INDEX, what
        assert bool((out == 7.0).all()), what        # the attention kernels did not run
    # entries past a sequence's last block are never looked at: -1 there is fine
    assert (wl.block_tables[1, 3:] == -1).all()
    attend(torch.from_numpy(wl.block_tables).cuda(), sl)
    assert attn_err(out.cpu().numpy(), want) <= 2e-3


def test_a_broken_shared_prefix_promise_is_reported(debug_on):
    """paged_decode_attn_prefix trusts the caller that the blocks below shared_prefix_tokens
    are the same in every table; the checks compare them with sequence 0's."""
    import torch
    from paper_2605_29639_amd import kvq
    from helpers import gpu_attention, upload_oracle_cache
    wl = W.custom("debug_prefix", W.MODE_INT8, [300, 256, 400], 1, 8, 2, 128, 16, seed=5,
                  shared_prefix=256)
    oc, osc = oracle_fill(wl)
    want = oracle.paged_decode_attn(wl.q, oc, osc, wl.mode, wl.block_tables, wl.seq_lens, 1, wl.sm_scale)
    cache, scales, desc = upload_oracle_cache(wl, oc, osc)
    got = gpu_attention(wl, cache, scales, desc, shared_prefix_tokens=256)
    assert attn_err(got, want) <= 2e-3
    # sequence 2 maps its fourth block elsewhere (a valid block, but not the shared one)
    other = int(wl.block_tables[2, 17])
    broken = _with(wl.block_tables, (2, 3), other)
    q = bits_to_bf16_tensor(wl.q)
    out = torch.full((3, 8, 128), 7.0, dtype=torch.float32, device="cuda")
    ws = kvq.alloc_workspace(desc, 3, 1, 8, wl.max_seq_len, shared_prefix_tokens=256)
    with pytest.raises(kvq.KvqError) as e:
        kvq.paged_decode_attn(q, cache, scales, desc, torch.from_numpy(broken).cuda(),
                              torch.from_numpy(wl.seq_lens).cuda(), 1, wl.max_seq_len, wl.sm_scale,
                              out, ws, shared_prefix_tokens=256)
    assert e.value.code == kvq.E_BAD_INDEX
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
    # the same tables without the promise are a valid call
    kvq.paged_decode_attn(q, cache, scales, desc, torch.from_numpy(broken).cuda(),
                          torch.from_numpy(wl.seq_lens).cuda(), 1, wl.max_seq_len, wl.sm_scale,
                          out, ws)
    torch.cuda.synchronize()
    assert np.isfinite(out.cpu().numpy()).all()


def _with(a, at, value):
    a = a.copy()
    a[at] = value
    return a
