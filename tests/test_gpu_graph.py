"""The entry points allocate nothing, keep no per-call state and never touch the host after
validation, so a decode step (kv_quant_write of the newest tokens + paged_decode_attn) can be
captured in a HIP graph once and replayed: the sequence lengths, tables, queries and new rows
are read on the device at every replay.  Each replay is checked bit for bit against the same
calls made eagerly on the same inputs, with eager work and synchronisations in between."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2605_29639_amd import workloads as W
from helpers import bits_to_bf16_tensor, gpu_fill


@pytest.mark.parametrize("mode", [W.MODE_INT8, W.MODE_FP8])
def test_a_captured_decode_step_replays_like_eager_calls(mode):
    import torch
    from paper_2605_29639_amd import kvq
    wl = W.custom("graph", mode, [200, 77, 1030, 64, 513], 1, 8, 2, 128, 16, seed=5)
    B, Hq, D, H = wl.batch, wl.num_q_heads, wl.head_dim, wl.num_kv_heads
    max_len = int(wl.seq_lens.max())
    bt = torch.from_numpy(wl.block_tables).cuda()
    rng = np.random.default_rng(77)

    def fresh_inputs(lens):
        """q, the newest token's k and v (random bf16) and its slot, for the given lengths."""
        q = W.to_bf16_bits(rng.standard_normal((B, Hq, D), dtype=np.float32))
        k = W.to_bf16_bits(rng.standard_normal((B, H, D), dtype=np.float32))
        v = W.to_bf16_bits(rng.standard_normal((B, H, D), dtype=np.float32))
        slots = np.array([wl.slots(b, int(lens[b]) - 1, int(lens[b]))[0] for b in range(B)], np.int64)
        return (bits_to_bf16_tensor(q), bits_to_bf16_tensor(k), bits_to_bf16_tensor(v),
                torch.from_numpy(slots).cuda(), torch.from_numpy(lens.astype(np.int32)).cuda())

    def step(cache, scales, desc, ins, out, ws):
        q, k, v, slots, sl = ins
        kvq.kv_quant_write(k, v, slots, cache, scales, desc)
        kvq.paged_decode_attn(q, cache, scales, desc, bt, sl, 1, max_len, wl.sm_scale, out, ws)

    # two identical caches: one for the graph, one for the eager calls
    cache_g, scales_g, desc = gpu_fill(wl)
    cache_e, scales_e = cache_g.clone(), scales_g.clone()
    ws_g = kvq.alloc_workspace(desc, B, 1, Hq, max_len, 0)
    ws_e = kvq.alloc_workspace(desc, B, 1, Hq, max_len, 0)
    out_g = torch.zeros((B, Hq, D), dtype=torch.float32, device="cuda")
    out_e = torch.zeros_like(out_g)

    static = fresh_inputs(wl.seq_lens)              # the tensors the graph reads
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                   # warm-up on the capture stream
        step(cache_g, scales_g, desc, static, out_g, ws_g)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    cache_g.copy_(cache_e), scales_g.copy_(scales_e)

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(cache_g, scales_g, desc, static, out_g, ws_g)
    cache_g.copy_(cache_e), scales_g.copy_(scales_e)   # (capturing runs nothing, but be sure)

    lens = wl.seq_lens.copy()
    for replay in range(4):
        if replay == 2:      # another decode position for two of the sequences
            lens[0] -= 37
            lens[2] -= 500
        new = fresh_inputs(lens)
        for dst, src in zip(static, new):
            dst.copy_(src)
        torch.cuda.synchronize()
        graph.replay()
        step(cache_e, scales_e, desc, new, out_e, ws_e)   # eager, same inputs
        torch.cuda.synchronize()
        assert torch.equal(out_g, out_e), "replay %d differs from the eager calls" % replay
        assert torch.equal(cache_g, cache_e) and torch.equal(scales_g, scales_e), replay
        assert torch.isfinite(out_g).all()


def test_a_captured_verify_step_with_a_shared_prefix_replays_like_eager_calls():
    """The same for paged_decode_attn_prefix (prefix kernel, streaming kernel, reduce): whether
    the prefix is used is decided on the device at every replay, so a replay in which one
    sequence has become shorter than the prefix falls back by itself."""
    import torch
    from paper_2605_29639_amd import kvq
    q_len, prefix = 4, 256
    wl = W.custom("graph_prefix", W.MODE_INT8, [700, 300, 1030, 260], q_len, 8, 2, 128, 16, seed=6,
                  shared_prefix=prefix)
    B, Hq, D, H = wl.batch, wl.num_q_heads, wl.head_dim, wl.num_kv_heads
    max_len = int(wl.seq_lens.max())
    bt = torch.from_numpy(wl.block_tables).cuda()
    rng = np.random.default_rng(78)

    def fresh_inputs(lens):
        q = W.to_bf16_bits(rng.standard_normal((B * q_len, Hq, D), dtype=np.float32))
        k = W.to_bf16_bits(rng.standard_normal((B * q_len, H, D), dtype=np.float32))
        v = W.to_bf16_bits(rng.standard_normal((B * q_len, H, D), dtype=np.float32))
        slots = np.concatenate([wl.slots(b, int(lens[b]) - q_len, int(lens[b])) for b in range(B)])
        return (bits_to_bf16_tensor(q), bits_to_bf16_tensor(k), bits_to_bf16_tensor(v),
                torch.from_numpy(slots.astype(np.int64)).cuda(),
                torch.from_numpy(lens.astype(np.int32)).cuda())

    def step(cache, scales, desc, ins, out, ws):
        q, k, v, slots, sl = ins
        kvq.kv_quant_write(k, v, slots, cache, scales, desc)
        kvq.paged_decode_attn(q, cache, scales, desc, bt, sl, q_len, max_len, wl.sm_scale, out, ws,
                              shared_prefix_tokens=prefix)

    cache_g, scales_g, desc = gpu_fill(wl)
    cache_e, scales_e = cache_g.clone(), scales_g.clone()
    ws_g = kvq.alloc_workspace(desc, B, q_len, Hq, max_len, 0, shared_prefix_tokens=prefix)
    ws_e = kvq.alloc_workspace(desc, B, q_len, Hq, max_len, 0, shared_prefix_tokens=prefix)
    out_g = torch.zeros((B * q_len, Hq, D), dtype=torch.float32, device="cuda")
    out_e = torch.zeros_like(out_g)

    static = fresh_inputs(wl.seq_lens)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(cache_g, scales_g, desc, static, out_g, ws_g)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    cache_g.copy_(cache_e), scales_g.copy_(scales_e)

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(cache_g, scales_g, desc, static, out_g, ws_g)
    cache_g.copy_(cache_e), scales_g.copy_(scales_e)

    lens = wl.seq_lens.copy()
    for replay in range(4):
        if replay == 1:      # other decode positions, every sequence still holds the prefix
            lens[0] -= 37
            lens[2] -= 500
        if replay == 2:      # sequence 3 shorter than the prefix: the prefix is not used
            lens[3] = 200
        if replay == 3:
            lens[3] = 256    # exactly the prefix: nothing but shared positions
        new = fresh_inputs(lens)
        for dst, src in zip(static, new):
            dst.copy_(src)
        torch.cuda.synchronize()
        graph.replay()
        step(cache_e, scales_e, desc, new, out_e, ws_e)
        torch.cuda.synchronize()
        assert torch.equal(out_g, out_e), "replay %d differs from the eager calls" % replay
        assert torch.equal(cache_g, cache_e) and torch.equal(scales_g, scales_e), replay
        assert torch.isfinite(out_g).all()
