"""paged_decode_attn_static: the entry point for callers that cannot allocate.  It runs the
kernels of paged_decode_attn on the library's own static scratch buffer, so its output must
equal paged_decode_attn's bit for bit; and since every call on a GPU shares that one buffer,
a second, smaller call right after a larger one must not be disturbed by what the first left."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2605_29639_amd import workloads as W
from helpers import bits_to_bf16_tensor, gpu_fill


def run_both(wl, cache, scales, desc, chunk):
    import torch
    from paper_2605_29639_amd import kvq
    q = bits_to_bf16_tensor(wl.q)
    bt = torch.from_numpy(wl.block_tables).cuda()
    sl = torch.from_numpy(wl.seq_lens).cuda()
    max_len = wl.max_seq_len
    shape = (wl.q.shape[0], wl.num_q_heads, wl.head_dim)
    want = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    got = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    ws = kvq.alloc_workspace(desc, wl.batch, wl.q_len, wl.num_q_heads, max_len, chunk)
    assert ws.numel() <= kvq.STATIC_WORKSPACE_BYTES
    kvq.paged_decode_attn(q, cache, scales, desc, bt, sl, wl.q_len, max_len, wl.sm_scale, want, ws,
                          chunk_tokens=chunk)
    kvq.paged_decode_attn_static(q, cache, scales, desc, bt, sl, wl.q_len, max_len, wl.sm_scale,
                                 got, chunk_tokens=chunk)
    torch.cuda.synchronize()
    return got.cpu().numpy(), want.cpu().numpy()


@pytest.mark.parametrize("mode", [W.MODE_INT8, W.MODE_FP8])
def test_static_scratch_equals_caller_workspace_twice_in_a_row(mode):
    import oracle
    from helpers import attn_err, oracle_fill
    big = W.custom("static_big", mode, [700, 64, 1500, 333, 65, 2049, 1, 900], 1, 8, 2, 128, 16,
                   seed=71 + mode)
    small = W.custom("static_small", mode, [130, 17], 1, 8, 2, 128, 16, seed=72 + mode)
    for wl, chunk in ((big, 0), (small, 64)):       # the second call is the smaller one
        cache, scales, desc = gpu_fill(wl)
        got, want = run_both(wl, cache, scales, desc, chunk)
        assert not np.isnan(got).any()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
        oc, osc = oracle_fill(wl)
        ref = oracle.paged_decode_attn(wl.q, oc, osc, wl.mode, wl.block_tables, wl.seq_lens,
                                       wl.q_len, wl.sm_scale)
        assert attn_err(got, ref) <= 2e-3
