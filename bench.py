"""Benchmark of the hot path on one MI355X: quantized paged decode attention, achieved HBM
GB/s and microseconds per layer, next to the CPU checker timed on the host cores.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--mode MODE]
                    [--configs all|none]

One step = one decode step of one layer over the whole batch: kv_quant_write of each
sequence's newest token(s), then paged_decode_attn over the layer's cache.  Successive steps
cycle through several layers' caches so that every step streams from HBM rather than from the
256 MB last-level cache.  Prints ONE JSON line: the headline workload (the Llama-3-8B-shaped
layer unless --workload says otherwise) at the top level, and under "configs" the same step
measured on the other benchmark configurations (fp8 + append, long context, verify + shared
prefix in both of its cache modes).

The step, the attention call and the write are timed through the library proper (libkvq.so).
The streaming kernel alone is timed through the measurement build of the same sources
(libkvq_prof.so), which can leave out the reduce so that a run of calls is a run of
back-to-back streaming kernels between two HIP events.
"""
import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, published peak
MFMA_F16_PEAK_TFLOPS = 2500.0

MODE_NAMES = {0: "int8", 1: "fp8", 2: "bf16", 3: "fp8_tensor", 4: "int4", 5: "int4_group"}
MODE_LONG = {0: "int8_token_head", 1: "fp8e4m3_block_head", 2: "bf16_unquantized",
             3: "fp8e4m3_static_tensor_scales", 4: "int4_token_head",
             5: "int4_scale_per_32_channels"}


class HipEvents:
    """Raw HIP events (ctypes over libamdhip64) recorded on the stream the kernels run on."""

    def __init__(self, stream):
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [C.c_void_p]
        self.hip.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        self.stream = C.c_void_p(stream)
        self.pool = []

    def create(self):
        e = C.c_void_p()
        assert self.hip.hipEventCreate(C.byref(e)) == 0
        return e

    def record(self, e):
        assert self.hip.hipEventRecord(e, self.stream) == 0

    def elapsed_ms(self, a, b):
        assert self.hip.hipEventSynchronize(b) == 0
        ms = C.c_float()
        assert self.hip.hipEventElapsedTime(C.byref(ms), a, b) == 0
        return ms.value

    def events(self, n):
        while len(self.pool) < n:
            self.pool.append(self.create())
        return self.pool[:n]


def measured_traffic(wl):
    """HBM bytes per launch of the streaming kernel for this workload from the committed
    rocprofv3 FETCH_SIZE / WRITE_SIZE summary (profiles/traffic.json), or None: counters cannot
    be read from inside this process, so the figure is as old as that file."""
    try:
        table = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))
        return table["%s/%s" % (wl.name, MODE_NAMES[wl.mode])]["hbm_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def make_workload(name, mode):
    from paper_2605_29639_amd import workloads as W
    kw = {} if mode is None else {"mode": {"int8": W.MODE_INT8, "fp8": W.MODE_FP8,
                                           "bf16": W.MODE_BF16,
                                           "fp8_tensor": W.MODE_FP8_TENSOR,
                                           "int4": W.MODE_INT4,
                                           "int4_group": W.MODE_INT4_GROUP}[mode]}
    makers = {"llama8b": W.llama8b, "fp8_append": W.fp8_append, "long_gqa": W.long_gqa,
              "verify_prefix": W.verify_prefix}
    if name not in makers:
        raise SystemExit("unknown workload %s" % name)
    return makers[name](**kw)


def percentiles(us):
    import numpy as np
    us = np.asarray(us, dtype=np.float64)
    return {"median": float(np.median(us)), "p10": float(np.percentile(us, 10)),
            "p90": float(np.percentile(us, 90)), "mean": float(us.mean())}


class Layers:
    """One workload resident in HBM: `n` layer caches (the library writes the first from the
    workload's rows; the others are device copies of it, which is all that cycling through
    distinct memory needs), queries, tables, the step's newest tokens, output, workspace."""

    def __init__(self, wl, n, chunk, alias_blocks=0):
        import numpy as np
        import torch
        from paper_2605_29639_amd import kvq
        from paper_2605_29639_amd.fill import bits_to_bf16_tensor, gpu_fill
        t0 = time.time()
        cache, scales, self.desc = gpu_fill(wl, workers=min(16, os.cpu_count() or 1))
        self.caches = [(cache, scales)] + [(cache.clone(), scales.clone()) for _ in range(n - 1)]
        self.setup_s = time.time() - t0
        self.wl, self.n, self.chunk = wl, n, chunk
        B = wl.batch
        self.q = bits_to_bf16_tensor(wl.q)
        bt = torch.from_numpy(wl.block_tables).cuda()
        if alias_blocks:
            bt = torch.where(bt >= 0, bt % alias_blocks, bt).contiguous()
        self.bt = bt
        self.sl = torch.from_numpy(wl.seq_lens).cuda()
        self.out = torch.empty((B * wl.q_len, wl.num_q_heads, wl.head_dim), dtype=torch.float32,
                               device="cuda")
        self.ws = kvq.alloc_workspace(self.desc, B, wl.q_len, wl.num_q_heads, wl.max_seq_len, chunk,
                                      shared_prefix_tokens=wl.shared_prefix)
        # the newest token(s) of every sequence: what a decode step appends before attending
        self.newest = [wl.kv_rows(b, int(wl.seq_lens[b]) - wl.q_len, int(wl.seq_lens[b]))
                       for b in range(B)]
        self.k_new = bits_to_bf16_tensor(np.concatenate([r[0] for r in self.newest]))
        self.v_new = bits_to_bf16_tensor(np.concatenate([r[1] for r in self.newest]))
        self.slots_new = torch.from_numpy(np.concatenate(
            [wl.slots(b, int(wl.seq_lens[b]) - wl.q_len, int(wl.seq_lens[b]))
             for b in range(B)])).cuda()
        self.stream = torch.cuda.current_stream().cuda_stream

    def write(self, i, L=None):
        from paper_2605_29639_amd import kvq
        cache, scales = self.caches[i % self.n]
        kvq.kv_quant_write(self.k_new, self.v_new, self.slots_new, cache, scales, self.desc,
                           stream=self.stream, L=L)

    def attn(self, i, L=None):
        from paper_2605_29639_amd import kvq
        wl = self.wl
        cache, scales = self.caches[i % self.n]
        kvq.paged_decode_attn(self.q, cache, scales, self.desc, self.bt, self.sl, wl.q_len,
                              wl.max_seq_len, wl.sm_scale, self.out, self.ws,
                              chunk_tokens=self.chunk, stream=self.stream, L=L,
                              shared_prefix_tokens=wl.shared_prefix)

    def step(self, i, L=None):
        self.write(i, L)
        self.attn(i, L)


def wall_us(fn, steps):
    """Mean microseconds per call of fn(i) over exactly `steps` calls, the device idle on both
    sides of the timed region."""
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        fn(i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps * 1e6


def event_spans_us(ev, fn, steps):
    """Per-call durations: an event after every call, each call's span taken between its
    neighbours' events (includes the event packets' own small cost)."""
    import torch
    marks = ev.events(steps + 1)
    torch.cuda.synchronize()
    ev.record(marks[0])
    for i in range(steps):
        fn(i)
        ev.record(marks[i + 1])
    torch.cuda.synchronize()
    return [ev.elapsed_ms(marks[i], marks[i + 1]) * 1e3 for i in range(steps)]


def bracket_us(ev, fn, steps):
    """Mean microseconds per call between one event ahead of and one behind `steps` calls."""
    import torch
    e0, e1 = ev.events(2)
    torch.cuda.synchronize()
    ev.record(e0)
    for i in range(steps):
        fn(i)
    ev.record(e1)
    torch.cuda.synchronize()
    return ev.elapsed_ms(e0, e1) * 1e3 / steps


def cpu_baseline(wl, newest, out_gpu, budget_tokens):
    """The CPU checker on the host cores, the same step on the first sequences of the workload
    (as many as fit `budget_tokens` stored tokens), median of 3; also the parity of the GPU's
    output with it on those sequences."""
    import numpy as np
    import oracle
    from helpers import oracle_fill
    from paper_2605_29639_amd.fill import attn_err
    B = wl.batch
    n_seq, tok = 0, 0
    while n_seq < B and (tok + int(wl.seq_lens[n_seq]) <= budget_tokens or n_seq == 0):
        tok += int(wl.seq_lens[n_seq])
        n_seq += 1
    seqs = list(range(n_seq))
    oc, osc = oracle_fill(wl, sequences=seqs)
    qs = np.ascontiguousarray(wl.q[:n_seq * wl.q_len])
    bts = np.ascontiguousarray(wl.block_tables[:n_seq])
    sls = np.ascontiguousarray(wl.seq_lens[:n_seq])
    ks = np.concatenate([n[0] for n in newest[:n_seq]])
    vs = np.concatenate([n[1] for n in newest[:n_seq]])
    ss = np.concatenate([wl.slots(b, int(wl.seq_lens[b]) - wl.q_len, int(wl.seq_lens[b]))
                         for b in seqs])
    times = []
    for _ in range(3):
        t0 = time.perf_counter()
        oracle.kv_quant_write(ks, vs, ss, oc, osc, wl.mode)
        want = oracle.paged_decode_attn(qs, oc, osc, wl.mode, bts, sls, wl.q_len, wl.sm_scale)
        times.append(time.perf_counter() - t0)
    cpu_s = float(np.median(times))
    alg = wl.algorithmic_bytes()
    frac = tok / float(wl.seq_lens.sum())
    base = {"value": alg["logical_total"] * frac / cpu_s / 1e9, "unit": "GB/s",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "first %d of %d sequences (%d of %d tokens), same step (write of the newest "
                      "tokens + attention), median of 3; %.3f s per sampled step"
                      % (n_seq, B, tok, int(wl.seq_lens.sum()), cpu_s),
            "us_per_layer_scaled_to_full": cpu_s / frac * 1e6}
    return base, attn_err(out_gpu[:n_seq * wl.q_len], want)


def measure(wl, args, ev, prof, cpu_budget_tokens):
    """Everything reported per workload.  Returns (result dict, Layers)."""
    import numpy as np
    import torch
    chunk = 0 if args.chunk < 0 else args.chunk
    alg = wl.algorithmic_bytes()
    # enough layer caches that the cycled live bytes exceed 4 x the 256 MB last-level cache
    n_layers = args.layers or max(2, int(np.ceil(4 * 256e6 / alg["kv"])))
    lay = Layers(wl, n_layers, chunk, args.alias_blocks)
    steps, warmup = args.steps, args.warmup

    # untimed: bring clocks and caches to their steady state (a fresh GPU needs a few hundred
    # milliseconds of load before kernel times settle), then the W warmup steps
    t_pre = time.perf_counter()
    while time.perf_counter() - t_pre < args.prewarm_s:
        for i in range(20):
            lay.step(i)
        torch.cuda.synchronize()
    for i in range(warmup):
        lay.step(i)
    step_us = wall_us(lay.step, steps)                 # the headline figure: exactly K steps
    step_spans = event_spans_us(ev, lay.step, steps)   # the same steps, one by one
    attn_us = wall_us(lay.attn, steps)
    attn_spans = event_spans_us(ev, lay.attn, steps)
    write_us = wall_us(lay.write, steps)

    # The dominant kernel alone: back-to-back launches of the streaming kernel between two
    # events on its stream (the measurement build leaves out the reduce); that span per launch
    # (end of the previous kernel to end of this one) is also what rocprofv3 reports per kernel.
    prof.kvq_profile_skip_reduce(1)
    try:
        for i in range(warmup):
            lay.attn(i, prof)
        kern_us = bracket_us(ev, lambda i: lay.attn(i, prof), steps)
    finally:
        prof.kvq_profile_skip_reduce(0)
    # the same access pattern with the arithmetic taken out (the read-ceiling twin)
    prof.kvq_profile_read_ceiling(1)
    try:
        for i in range(warmup):
            lay.attn(i, prof)
        ceil_us = bracket_us(ev, lambda i: lay.attn(i, prof), steps)
    finally:
        prof.kvq_profile_read_ceiling(0)
    # cross-check: the attention call through the measurement build (all switches off) must
    # cost what it costs through the library proper
    attn_prof_us = wall_us(lambda i: lay.attn(i, prof), steps)

    lay.step(1)
    torch.cuda.synchronize()
    out_gpu = lay.out.cpu().numpy()

    gbps = lambda us: alg["total"] / us / 1e3
    res = {
        "config": {"workload": wl.name, "mode": MODE_LONG[wl.mode], "batch": wl.batch,
                   "q_len": wl.q_len, "num_q_heads": wl.num_q_heads,
                   "num_kv_heads": wl.num_kv_heads, "head_dim": wl.head_dim,
                   "block_size": wl.block_size, "sum_seq_lens": int(wl.seq_lens.sum()),
                   "max_seq_len": wl.max_seq_len, "shared_prefix_tokens": wl.shared_prefix,
                   "chunk_tokens": chunk or "auto (even split over the resident wavefronts)",
                   "layers_cycled": n_layers,
                   "step": "kv_quant_write(newest token%s) + paged_decode_attn"
                           % ("s" if wl.q_len > 1 else "")},
        "value": gbps(step_us), "unit": "GB/s",
        "us_per_layer": step_us,
        "us_per_layer_by_step": percentiles(step_spans),
        "pct_of_hbm_peak": 100.0 * gbps(step_us) / HBM_PEAK_GBPS,
        "attn_only_us_per_layer": attn_us,
        "attn_only_us_by_call": percentiles(attn_spans),
        "attn_only_pct_of_hbm_peak": 100.0 * gbps(attn_us) / HBM_PEAK_GBPS,
        "attn_only_us_through_measurement_build": attn_prof_us,
        "write_only_us_per_layer": write_us,
        "algorithmic_bytes": alg,
        "roofline": {"bound": "hbm", "kernel": "attn_stream_kernel",
                     "achieved": gbps(kern_us), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": gbps(kern_us) / HBM_PEAK_GBPS,
                     "traffic": measured_traffic(wl),
                     "traffic_source": "profiles/traffic.json (rocprofv3 counter runs; not "
                                       "measured in this run)",
                     "kernel_us_mean": kern_us,
                     "read_ceiling_us": ceil_us,
                     "read_ceiling_gbps": gbps(ceil_us),
                     "frac_of_read_ceiling": ceil_us / kern_us,
                     # the operation the caller sees: streaming kernel + reduce, and the step
                     "call_us": attn_us, "call_frac": gbps(attn_us) / HBM_PEAK_GBPS,
                     "step_us": step_us, "step_frac": gbps(step_us) / HBM_PEAK_GBPS},
        "setup_s": lay.setup_s,
    }
    if not args.no_cpu_baseline:
        res["cpu_baseline"], res["parity_vs_oracle_on_sample"] = cpu_baseline(
            wl, lay.newest, out_gpu, cpu_budget_tokens)
    return res, lay, out_gpu


def extras(res, lay, out_main, args, ev, prof):
    """Reported for the headline workload only: the prompt-sized write, block moves, a chunk of
    a prompt through the same entry point, and the same step over an unquantized cache."""
    import numpy as np
    import torch
    from paper_2605_29639_amd import kvq, workloads as Wm
    from paper_2605_29639_amd.fill import attn_err, bits_to_bf16_tensor, gpu_fill
    wl, desc, stream = lay.wl, lay.desc, lay.stream
    B, Hq, D = wl.batch, wl.num_q_heads, wl.head_dim

    # Bulk (prompt-sized) kv_quant_write: the first sequences' tokens, at least 32k of them, in
    # one call, rewritten into the first layer cache.  Bytes = bf16 rows read + codes and
    # scales written.
    n_seq, n_tok = 0, 0
    while n_seq < B and n_tok < 32768:
        n_tok += wl.write_range(n_seq)[1] - wl.write_range(n_seq)[0]
        n_seq += 1
    rows = [wl.kv_rows(b, *wl.write_range(b)) for b in range(n_seq)]
    k_bulk = bits_to_bf16_tensor(np.concatenate([r[0] for r in rows]))
    v_bulk = bits_to_bf16_tensor(np.concatenate([r[1] for r in rows]))
    s_bulk = torch.from_numpy(np.concatenate(
        [wl.slots(b, *wl.write_range(b)) for b in range(n_seq)])).cuda()
    del rows
    cache0, scales0 = lay.caches[0]
    bulk = lambda i: kvq.kv_quant_write(k_bulk, v_bulk, s_bulk, cache0, scales0, desc, stream=stream)
    for i in range(3):
        bulk(i)
    bulk_us = bracket_us(ev, bulk, 10)
    per_row = 2 * D + {0: D + 4, 1: D + 4.0 / wl.block_size, 2: 2 * D, 3: D, 4: D / 2 + 4,
                       5: D / 2 + D / 8}[wl.mode]
    bulk_bytes = n_tok * wl.num_kv_heads * 2 * per_row
    res["prefill_write"] = {"tokens": n_tok, "sequences": n_seq, "us": bulk_us,
                            "bytes": bulk_bytes, "GB/s": bulk_bytes / bulk_us / 1e3,
                            "frac_of_hbm_peak": bulk_bytes / bulk_us / 1e3 / HBM_PEAK_GBPS,
                            "tokens_per_s": n_tok / bulk_us * 1e6}
    del k_bulk, v_bulk, s_bulk

    # Block moves between the pool and a packed staging area (the tiered cache's load and evict
    # steps): about 64 MB of blocks of the second layer cache, to and from device memory and
    # pinned host memory.  GB/s counts the bytes once (they are read once and written once).
    cache1, scales1 = lay.caches[1 % lay.n]
    n_blk = int(min(desc.num_blocks, max(1, (64 << 20) // kvq.packed_sizes(desc, 1)[0])))
    ids = torch.from_numpy(np.random.default_rng(1).permutation(desc.num_blocks)[:n_blk]
                           .astype(np.int32)).cuda()
    cb, sf = kvq.packed_sizes(desc, n_blk)
    moves = {"blocks": n_blk, "bytes": cb + 4 * sf}
    for where, kw in (("device", dict(device="cuda")), ("pinned_host", dict(pin_memory=True))):
        pc = torch.empty(cb, dtype=torch.uint8, **kw)
        ps = torch.empty(sf, dtype=torch.float32, **kw)
        for name, fn in (("export", lambda i: kvq.blocks_export(cache1, scales1, desc, ids, pc, ps, stream=stream)),
                         ("import", lambda i: kvq.blocks_import(pc, ps, desc, ids, cache1, scales1, stream=stream))):
            fn(0)
            us = bracket_us(ev, fn, 5)
            moves["%s_%s" % (name, where)] = {"us": us, "GB/s": (cb + 4 * sf) / us / 1e3}
        del pc, ps
    res["block_moves"] = moves

    # A chunk of a prompt through the same entry point: 512 query tokens per sequence attending
    # causally over a 4096-token prefix already in the cache and over themselves, 8 sequences,
    # this workload's heads and cache mode.  Useful flops = 4 * head_dim per (query row, visible
    # position); the bound here is the matrix cores, not HBM.
    cq, cL, cB = 512, 4608, 8
    wlc = Wm.chunk_prefill(wl.mode, batch=cB, chunk=cq, prefix=cL - cq, Hq=Hq, Hkv=wl.num_kv_heads,
                           D=D, bs=wl.block_size)
    cc, cs, cdesc = gpu_fill(wlc)
    qc = bits_to_bf16_tensor(wlc.q)
    btc = torch.from_numpy(wlc.block_tables).cuda()
    slc = torch.from_numpy(wlc.seq_lens).cuda()
    outc = torch.empty((cB * cq, Hq, D), dtype=torch.float32, device="cuda")
    wsc = kvq.alloc_workspace(cdesc, cB, cq, Hq, cL, 0)
    call = lambda i, L=None: kvq.paged_decode_attn(qc, cc, cs, cdesc, btc, slc, cq, cL, wlc.sm_scale,
                                                   outc, wsc, stream=stream, L=L)
    for i in range(3):
        call(i)
    chunk_us = bracket_us(ev, call, 10)
    prof.kvq_profile_prefill_kernel(0)  # the same call through the streaming kernels, for comparison
    try:
        call(0, prof)
        chunk_stream_us = bracket_us(ev, lambda i: call(i, prof), 5)
    finally:
        prof.kvq_profile_prefill_kernel(1)
    visible = sum(cL - cq + j + 1 for j in range(cq))
    tflops = 4.0 * D * Hq * cB * visible / chunk_us / 1e6
    res["chunk_prefill"] = {"sequences": cB, "chunk_tokens": cq, "context": cL, "us": chunk_us,
                            "us_through_streaming_kernels": chunk_stream_us,
                            "roofline": {"bound": "mfma", "kernel": "attn_prefill_kernel",
                                         "achieved": tflops, "peak": MFMA_F16_PEAK_TFLOPS,
                                         "unit": "TFLOP/s", "frac": tflops / MFMA_F16_PEAK_TFLOPS}}
    if wl.mode != 2 and not args.no_bf16_baseline:   # the same chunk over an unquantized cache
        wlb = Wm.chunk_prefill(2, batch=cB, chunk=cq, prefix=cL - cq, Hq=Hq, Hkv=wl.num_kv_heads,
                               D=D, bs=wl.block_size)
        cb_, sb_, bdesc = gpu_fill(wlb)
        wsb = kvq.alloc_workspace(bdesc, cB, cq, Hq, cL, 0)
        btb = torch.from_numpy(wlb.block_tables).cuda()
        callb = lambda i: kvq.paged_decode_attn(qc, cb_, sb_, bdesc, btb, slc, cq, cL, wlb.sm_scale,
                                                outc, wsb, stream=stream)
        for i in range(3):
            callb(i)
        chunk_bf16_us = bracket_us(ev, callb, 10)
        res["chunk_prefill"]["us_bf16_cache"] = chunk_bf16_us
        res["chunk_prefill"]["time_ratio_quantized_to_bf16"] = chunk_us / chunk_bf16_us
        del cb_, sb_, wsb, btb
    del cc, cs, qc, outc, wsc

    # The same step over an unquantized cache (the paper's Section 8.5 baseline): same shapes,
    # lengths, tables and K/V values, the rows stored as bf16.  The ratio is the kernel-level
    # form of the paper's claim that the quantized cache relieves decode of half its traffic.
    if wl.mode != 2 and not args.no_bf16_baseline:
        step_us, kern_us = res["us_per_layer"], res["roofline"]["kernel_us_mean"]
        q, bt, sl, out = lay.q, lay.bt, lay.sl, lay.out
        k_new, v_new, slots_new = lay.k_new, lay.v_new, lay.slots_new
        lay.caches = None
        torch.cuda.empty_cache()
        wl2 = make_workload(args.workload, "bf16")
        alg2 = wl2.algorithmic_bytes()
        lay2 = Layers(wl2, args.layers or max(2, int(np.ceil(4 * 256e6 / alg2["kv"]))),
                      lay.chunk, args.alias_blocks)
        for i in range(args.warmup + 20):
            lay2.step(i)
        step2_us = wall_us(lay2.step, args.steps)
        prof.kvq_profile_skip_reduce(1)
        try:
            for i in range(args.warmup):
                lay2.attn(i, prof)
            kern2_us = bracket_us(ev, lambda i: lay2.attn(i, prof), args.steps)
        finally:
            prof.kvq_profile_skip_reduce(0)
        lay2.step(1)
        torch.cuda.synchronize()
        res["bf16_baseline"] = {
            "us_per_layer": step2_us, "kernel_us_mean": kern2_us,
            "algorithmic_bytes": alg2["total"], "GB/s": alg2["total"] / step2_us / 1e3,
            "kernel_GB/s": alg2["total"] / kern2_us / 1e3,
            "step_time_ratio_quantized_to_bf16": step_us / step2_us,
            "kernel_time_ratio_quantized_to_bf16": kern_us / kern2_us,
            "bytes_ratio_quantized_to_bf16": res["algorithmic_bytes"]["total"] / alg2["total"],
            # how far quantization moves the output on this synthetic data (1 % of the K
            # channels are 20x outliers): max |quantized - bf16| / max |bf16|
            "output_deviation_quantized_vs_bf16":
                attn_err(out_main, lay2.out.cpu().numpy().astype(np.float64))}
        del lay2
        torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--prewarm-s", type=float, default=0.5,
                    help="seconds of untimed load before the warmup steps")
    ap.add_argument("--workload", default="llama8b",
                    help="the headline workload: llama8b, fp8_append, long_gqa or verify_prefix")
    ap.add_argument("--mode", default=None, choices=["int8", "fp8", "bf16", "fp8_tensor", "int4", "int4_group"],
                    help="override the headline workload's cache mode (bf16 = the unquantized baseline)")
    ap.add_argument("--configs", default=None, choices=["all", "none"],
                    help="also measure the other benchmark configurations (default: all when "
                         "the headline is the default one, else none)")
    ap.add_argument("--layers", type=int, default=0, help="layer caches cycled (0 = auto)")
    ap.add_argument("--chunk", type=int, default=-1, help="split-K granule in tokens (-1 or 0 = automatic)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-bf16-baseline", action="store_true",
                    help="skip timing the same workload over an unquantized (bf16) cache")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the prompt-sized write, block moves, prompt chunk and bf16 baseline")
    ap.add_argument("--alias-blocks", type=int, default=0,
                    help="diagnostic: fold every block-table entry modulo this many blocks so that "
                         "all reads hit the caches (shows the kernel's pure issue time); the "
                         "result line is then not a valid measurement")
    ap.add_argument("--calibrate-copy-mib", type=int, default=0,
                    help="also run plain device-to-device copies of this many MiB (a known-size "
                         "reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("this build measures one GPU only: run with --gpus 1 "
                         "(no collectives or sharding are part of it)")

    import torch
    from paper_2605_29639_amd import kvq
    kvq.lib()            # fails loudly if the HIP library is not built
    prof = kvq.prof_lib()
    torch.cuda.set_device(0)
    ev = HipEvents(torch.cuda.current_stream().cuda_stream)
    t_start = time.time()

    wl = make_workload(args.workload, args.mode)
    head, lay, out_main = measure(wl, args, ev, prof, cpu_budget_tokens=160000)
    if not args.no_extras:
        extras(head, lay, out_main, args, ev, prof)
    del lay
    torch.cuda.empty_cache()

    if args.calibrate_copy_mib:
        src = torch.empty(args.calibrate_copy_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        src.fill_(1)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    result = {
        "metric": "quantized paged decode attention: achieved HBM GB/s",
        "value": head["value"], "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["us_per_layer"] * 1e-3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.mode == 2 else "f16",   # the matrix instructions' operand type
        "dtype_detail": ("bf16 rows, bf16 MFMA operands, f32 accumulate and softmax" if wl.mode == 2 else
                         "u4 codes, f16 MFMA operands, f32 accumulate and softmax" if wl.mode in (4, 5) else
                         "u8 codes, f16 MFMA operands, f32 accumulate and softmax"),
        "data": "synthetic" if not args.alias_blocks else "INVALID: aliased block tables (diagnostic)",
    }
    result.update({k: v for k, v in head.items() if k not in ("value", "unit")})

    which = args.configs or ("all" if (args.workload == "llama8b" and args.mode is None) else "none")
    if which == "all":
        # the other benchmark configurations, the same step and the same measurements; the CPU
        # checker's sample is smaller for the block-scaled fp8 cache, which it fills slowly
        result["configs"] = []
        for name, mode, budget in (("fp8_append", None, 24000), ("long_gqa", None, 70000),
                                   ("verify_prefix", "int8", 60000), ("verify_prefix", "fp8", 24000)):
            r, lay, _ = measure(make_workload(name, mode), args, ev, prof, cpu_budget_tokens=budget)
            del lay
            torch.cuda.empty_cache()
            result["configs"].append(r)
    result["bench_wall_s"] = time.time() - t_start
    print(json.dumps(result))


if __name__ == "__main__":
    main()
