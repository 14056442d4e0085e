#!/usr/bin/env python3
"""Benchmark of the TokenRing per-device compute path on one MI355X.

One JSON line on stdout.  A *step* is one iteration of Algorithm 1 on one device at the
4096 x 4096, 32-head, D=128 block shape: tr_block_attn (bf16 block_out + fp32 block_lse)
followed by tr_merge of that block into the fp32 accumulators.  `value` is the step's
attention TFLOP (4*Sq*Sk*D per head) divided by the whole step time, inputs resident in
HBM.  `roofline` is the block-attention kernel against the bf16 MFMA peak, from HIP events
carried by every launch of a second pass over the same K steps right after the timed one (a
launch that carries events costs the host more, which is not the step's cost);
`merge_roofline` is the same for the merge kernel against HBM.  `parity` holds the max-abs errors of the same step against the
fp64 oracle on four heads.  `extras` adds the library GEMM's rate on this machine, the fused
step, the block step on other score distributions, the merge-only bandwidth workload
(pairwise and n-ary), the ring-schedule workloads and oracle timings of the other
workloads.  `cpu_baseline` times the fp64 oracle on heads of the same block step on the
host cores.

Before the warm-up steps the step runs untimed for about half a second: an idle MI355X needs
a few hundred milliseconds of load to leave its low-power clock state (rocm-smi shows the
shader clock climbing over that time), and a ring schedule keeps the device busy for far
longer than that, so the sustained state is the one to measure.  --no-ramp skips it.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "traffic.json")


def _traffic(kernel):
    """HBM bytes per launch of a kernel of the cfg2 step, from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs that
    profiles/traffic.json records (counters cannot be read from inside this process); None if not recorded."""
    try:
        with open(TRAFFIC_JSON) as f:
            return int(json.load(f)[kernel]["hbm_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        return None


def _settle(fn, seconds=0.25):
    """Untimed: runs the workload itself for a moment, so that what is timed next does not inherit the clock
    state the previous workload left (a library GEMM leaves the chip slower for tens of milliseconds)."""
    import torch
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(20):
            fn()
        torch.cuda.synchronize()


def _median(xs):
    xs = sorted(xs)
    n = len(xs)
    return xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])


def _dev(bits):
    import numpy as np
    import torch
    return torch.from_numpy(bits.view(np.int16)).to("cuda").view(torch.bfloat16)


def _event_ms(pairs):
    return [a.elapsed_time(b) for a, b in pairs]


def bench_block_step(tr, wl, steps, warmup, ramp_s):
    import numpy as np
    import torch
    cfg = wl.CONFIGS["cfg2_block"]
    qb, kb, vb = wl.make_qkv_bits(cfg)
    q, k, v = _dev(qb), _dev(kb), _dev(vb)
    B, H, S, D = cfg.B, cfg.Hq, cfg.S, cfg.D
    blk_o = torch.empty((B, H, S, D), dtype=torch.bfloat16, device="cuda")
    blk_l = torch.empty((B, H, S), dtype=torch.float32, device="cuda")
    acc_o = torch.zeros((B, H, S, D), dtype=torch.float32, device="cuda")
    acc_l = torch.full((B, H, S), float("-inf"), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    # Per-kernel durations: each launch carries its own start/stop HIP events in the dispatch
    # (tr_time_next_kernel), on the stream the kernels run on, so the event pair brackets the
    # kernel alone; the whole step is timed by the host clock around the K steps.
    def step(ev=None):
        if ev is not None:
            tr.tr_time_next_kernel(ev[0], ev[1])
        tr.tr_block_attn(q, k, v, tr.TR_MASK_NONE, cfg.scale, blk_o, blk_l, stream)
        if ev is not None:
            tr.tr_time_next_kernel(ev[2], ev[3])
        tr.tr_merge(acc_o, acc_l, blk_o, blk_l, stream)

    # parity of exactly this step (first one: the accumulators start as the identity of the Update) on four heads
    import oracle
    step()
    torch.cuda.synchronize()
    heads = [0, 13, 22, 31]
    err = {"block_out": 0.0, "block_lse": 0.0, "acc_out": 0.0, "acc_lse": 0.0}
    f = wl.bf16_bits_to_f64
    for h in heads:
        ref_o, ref_l = oracle.attention_block(f(qb[:, h:h + 1]), f(kb[:, h:h + 1]), f(vb[:, h:h + 1]), cfg.scale)
        d = lambda t, ref: float(np.max(np.abs(t.float().cpu().numpy().astype(np.float64) - ref)))
        err["block_out"] = max(err["block_out"], d(blk_o[:, h:h + 1], ref_o))
        err["block_lse"] = max(err["block_lse"], d(blk_l[:, h:h + 1], ref_l))
        err["acc_out"] = max(err["acc_out"], d(acc_o[:, h:h + 1], ref_o))      # Update of the identity with the block
        err["acc_lse"] = max(err["acc_lse"], d(acc_l[:, h:h + 1], ref_l))
    parity = {"against": "fp64 oracle, heads %s of the timed step in full" % heads, "max_abs": err,
              "tolerance": {"out": 1e-2, "lse": 1e-3}, "ok": bool(max(err["block_out"], err["acc_out"]) <= 1e-2 and
                                                                max(err["block_lse"], err["acc_lse"]) <= 1e-3)}

    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < ramp_s:      # untimed: lets the device reach its sustained clock state
        for _ in range(50):
            step()
        torch.cuda.synchronize()
    for _ in range(warmup):
        step()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    for evs in events:          # make torch create the handles (a first record) outside the timed regions
        for e in evs:
            e.record(stream)
    # The timed region: exactly K steps as a caller runs them, host clock between two synchronisations.
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    # The same K steps once more, every launch carrying its own event pair, for the kernel durations:
    # a dispatch with events costs about 5 us more on the host side (11 us per step, 4 %), which
    # would otherwise be charged to the step.
    t0 = time.perf_counter()
    for i in range(steps):
        step(events[i])
    torch.cuda.synchronize()
    ms_per_step_events = (time.perf_counter() - t0) * 1e3 / steps
    attn_ms = _event_ms([(e[0], e[1]) for e in events])
    merge_ms = _event_ms([(e[2], e[3]) for e in events])
    attn_avg, merge_avg = sum(attn_ms) / steps, sum(merge_ms) / steps
    flops = 4.0 * S * S * D * H * B                              # algorithmic: 4*D per (q,k) pair
    merge_bytes = B * H * S * (D * (4 + 2 + 4) + 3 * 4)          # read acc fp32 + block bf16, write acc; 3 lse words
    return {
        "cfg": cfg, "ms_per_step": ms_per_step, "ms_per_step_events": ms_per_step_events, "flops": flops, "parity": parity,
        "attn_ms_avg": attn_avg, "attn_ms_median": _median(attn_ms), "attn_ms_min": min(attn_ms),
        "merge_ms_avg": merge_avg, "merge_ms_median": _median(merge_ms), "merge_ms_min": min(merge_ms),
        "attn_tflops": flops / (attn_avg * 1e-3) / 1e12,
        "merge_gbs": merge_bytes / (merge_avg * 1e-3) / 1e9, "merge_bytes": merge_bytes,
    }


def bench_ring_small(tr, wl):
    """cfg1 (launch-bound correctness workload, 16 block steps of 64 x 64): time only, eager launches and as a HIP graph."""
    import torch
    cfg = wl.CONFIGS["cfg1_small"]
    qb, kb, vb = wl.make_qkv_bits(cfg)
    q, k, v = _dev(qb), _dev(kb), _dev(vb)
    out = torch.empty((cfg.B, cfg.Hq, cfg.S, cfg.D), dtype=torch.float32, device="cuda")
    lse = torch.empty((cfg.B, cfg.Hq, cfg.S), dtype=torch.float32, device="cuda")
    run = lambda: tr.tr_ring_attn(q, k, v, cfg.n_chunks, cfg.causal, out, lse, cfg.scale, None)

    def timed(fn, n=200):
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e6 / n

    eager_us = timed(run)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    graph_us = timed(graph.replay)
    return {"workload": "cfg1: B1 H2 S256 D64 as 4 chunks, non-causal, 16 block steps (launch-bound)",
            "us_eager": eager_us, "us_graph_replay": graph_us}


def bench_gemm_ceiling():
    """The library GEMM (torch.matmul on bf16 N(0,1) operands, 8192 x 8192 x 8192, fp32 accumulation) on this machine:
    an MFMA rate sustained by code that is not this repository's, next to which the attention kernel's can be read."""
    import torch
    n = 8192
    g = torch.Generator(device="cuda").manual_seed(20501)
    a = torch.randn((n, n), dtype=torch.float32, device="cuda", generator=g).to(torch.bfloat16)
    b = torch.randn((n, n), dtype=torch.float32, device="cuda", generator=g).to(torch.bfloat16)
    c = torch.empty((n, n), dtype=torch.bfloat16, device="cuda")
    for _ in range(5):
        torch.matmul(a, b.t(), out=c)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
    for x, y in ev:
        x.record(); torch.matmul(a, b.t(), out=c); y.record()
    torch.cuda.synchronize()
    ms = sorted(_event_ms(ev))
    flop = 2.0 * n ** 3
    med = ms[len(ms) // 2]
    return {"workload": "torch.matmul bf16 N(0,1) 8192^3 (A row-major, B transposed), library GEMM", "ms_median": med,
            "tflops": flop / (med * 1e-3) / 1e12, "frac_mfma_peak": flop / (med * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "tflops_best": flop / (ms[0] * 1e-3) / 1e12}


def bench_step_fused(tr, wl, steps, warmup):
    """The same block step as one kernel: tr_block_attn_merge (Update applied in the attention epilogue)."""
    import torch
    cfg = wl.CONFIGS["cfg2_block"]
    qb, kb, vb = wl.make_qkv_bits(cfg)
    q, k, v = _dev(qb), _dev(kb), _dev(vb)
    acc_o = torch.zeros((cfg.B, cfg.Hq, cfg.S, cfg.D), dtype=torch.float32, device="cuda")
    acc_l = torch.full((cfg.B, cfg.Hq, cfg.S), float("-inf"), dtype=torch.float32, device="cuda")
    _settle(lambda: tr.tr_block_attn_merge(q, k, v, tr.TR_MASK_NONE, cfg.scale, acc_o, acc_l))
    for _ in range(warmup):
        tr.tr_block_attn_merge(q, k, v, tr.TR_MASK_NONE, cfg.scale, acc_o, acc_l)
    torch.cuda.synchronize()
    t0 = time.perf_counter()                 # the step as a caller runs it: host clock over back-to-back launches
    for _ in range(steps):
        tr.tr_block_attn_merge(q, k, v, tr.TR_MASK_NONE, cfg.scale, acc_o, acc_l)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in ev:
        a.record(); b.record()
    for a, b in ev:                          # the kernel alone
        tr.tr_time_next_kernel(a, b)
        tr.tr_block_attn_merge(q, k, v, tr.TR_MASK_NONE, cfg.scale, acc_o, acc_l)
    torch.cuda.synchronize()
    kernel_ms = _median(_event_ms(ev))
    flops = 4.0 * cfg.S * cfg.S * cfg.D * cfg.Hq * cfg.B
    return {"workload": "cfg2 block step as one kernel (tr_block_attn_merge)", "ms": ms, "kernel_ms_median": kernel_ms,
            "tflops": flops / (ms * 1e-3) / 1e12, "frac_mfma_peak": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}


def bench_block(tr, wl, name, steps, warmup, what):
    """One block step (bf16 block_out) of a named 4096 x 4096 workload: diagonal-causal, or another score distribution."""
    import torch
    cfg = wl.CONFIGS[name]
    qb, kb, vb = wl.make_qkv_bits(cfg)
    q, k, v = _dev(qb), _dev(kb), _dev(vb)
    blk_o = torch.empty((cfg.B, cfg.Hq, cfg.S, cfg.D), dtype=torch.bfloat16, device="cuda")
    blk_l = torch.empty((cfg.B, cfg.Hq, cfg.S), dtype=torch.float32, device="cuda")
    mask = tr.TR_MASK_CAUSAL_DIAG if cfg.causal else tr.TR_MASK_NONE
    _settle(lambda: tr.tr_block_attn(q, k, v, mask, cfg.scale, blk_o, blk_l))
    for _ in range(warmup):
        tr.tr_block_attn(q, k, v, mask, cfg.scale, blk_o, blk_l)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a_, b_ in ev:
        tr.tr_time_next_kernel(a_, b_); tr.tr_block_attn(q, k, v, mask, cfg.scale, blk_o, blk_l)
    torch.cuda.synchronize()
    ms = _median(_event_ms(ev))
    flops = (2.0 * cfg.S * (cfg.S + 1) if cfg.causal else 4.0 * cfg.S * cfg.S) * cfg.D * cfg.Hq * cfg.B
    return {"workload": what, "ms_median": ms, "tflops": flops / (ms * 1e-3) / 1e12,
            "frac_mfma_peak": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}


def bench_merge_only(tr, wl, steps, warmup):
    """Eight fp32 partials [1,32,32768,128] merged in ring order (device-generated N(0,1) / U(-5,15))."""
    import torch
    cfg = wl.CONFIGS["cfg4_merge"]
    g = torch.Generator(device="cuda").manual_seed(cfg.seed)
    shape = (cfg.B, cfg.H, cfg.S, cfg.D)
    outs = [torch.randn(shape, dtype=torch.float32, device="cuda", generator=g) for _ in range(cfg.n_partials)]
    lses = [torch.rand(shape[:3], dtype=torch.float32, device="cuda", generator=g) * (cfg.lse_hi - cfg.lse_lo) + cfg.lse_lo
            for _ in range(cfg.n_partials)]
    acc_o = torch.zeros(shape, dtype=torch.float32, device="cuda")
    acc_l = torch.full(shape[:3], float("-inf"), dtype=torch.float32, device="cuda")
    per_call_bytes = 3 * (acc_o.numel() + acc_l.numel()) * 4
    for _ in range(warmup):
        tr.tr_merge(acc_o, acc_l, outs[0], lses[0])
    durations = []
    for _ in range(steps):
        acc_o.zero_(); acc_l.fill_(float("-inf"))
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(cfg.n_partials)]
        for i, (a, b) in enumerate(ev):
            tr.tr_time_next_kernel(a, b); tr.tr_merge(acc_o, acc_l, outs[i], lses[i])
        torch.cuda.synchronize()
        durations += _event_ms(ev)
    ms = sum(durations) / len(durations)
    gbs = per_call_bytes / (ms * 1e-3) / 1e9
    res = {"workload": "cfg4 merge-only: 8 fp32 partials [1,32,32768,128] in ring order", "ms_per_merge": ms,
           "bytes_per_merge": per_call_bytes, "gbs": gbs, "frac_hbm_peak": gbs / PEAK_HBM_GBS,
           "ms_all_8": ms * cfg.n_partials}
    # the same eight partials through one tr_merge_n call: each partial read once, result written once
    nary_bytes = (cfg.n_partials + 1) * (acc_o.numel() + acc_l.numel()) * 4
    tr.tr_merge_n(acc_o, acc_l, outs, lses)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(max(steps, 3))]
    for a, b in ev:
        tr.tr_time_next_kernel(a, b); tr.tr_merge_n(acc_o, acc_l, outs, lses)
    torch.cuda.synchronize()
    ms_n = sum(_event_ms(ev)) / len(ev)
    res["nary"] = {"ms_all_8": ms_n, "bytes": nary_bytes, "gbs": nary_bytes / (ms_n * 1e-3) / 1e9,
                   "frac_hbm_peak": nary_bytes / (ms_n * 1e-3) / 1e9 / PEAK_HBM_GBS}
    return res


def bench_ring(tr, wl, name, steps, warmup, fused, schedule=None, n_inner=1, block_dtype=None):
    """tr_ring_attn over a whole sequence; fused: Update in the attention epilogue (no workspace), else two kernels.
    schedule: None = tr_ring_attn (Algorithm 1), else a TR_SCHED_* value run through tr_ring_attn_sched."""
    import torch
    cfg = wl.CONFIGS[name]
    g = torch.Generator(device="cuda").manual_seed(cfg.seed)
    mk = lambda h: (torch.randn((cfg.B, h, cfg.S, cfg.D), dtype=torch.float32, device="cuda", generator=g) * cfg.std).to(torch.bfloat16)
    q, k, v = mk(cfg.Hq), mk(cfg.Hkv), mk(cfg.Hkv)
    out = torch.empty((cfg.B, cfg.Hq, cfg.S, cfg.D), dtype=torch.float32, device="cuda")
    lse = torch.empty((cfg.B, cfg.Hq, cfg.S), dtype=torch.float32, device="cuda")
    ws = None if fused else torch.empty(tr.tr_ring_attn_workspace_bytes(q, cfg.n_chunks), dtype=torch.uint8, device="cuda")

    def run():
        if block_dtype is not None:     # two-kernel form with a chosen transport format of block_out
            tr.tr_ring_attn_blocks(q, k, v, cfg.n_chunks, cfg.causal, out, lse, block_dtype, ws, cfg.scale)
        elif schedule is None:
            tr.tr_ring_attn(q, k, v, cfg.n_chunks, cfg.causal, out, lse, cfg.scale, ws)
        else:
            tr.tr_ring_attn_sched(q, k, v, cfg.n_chunks, cfg.causal, schedule, out, lse, cfg.scale, n_inner)

    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    n, C = cfg.n_chunks, cfg.chunk
    if schedule == tr.TR_SCHED_ZIGZAG:      # 2n segments of half the length
        n, C = 2 * n, C // 2
    full_steps = n * (n - 1) // 2 if cfg.causal else n * n
    diag_steps = n if cfg.causal else 0
    flops = cfg.B * cfg.Hq * cfg.D * (4.0 * C * C * full_steps + 2.0 * C * (C + 1) * diag_steps)
    sched_name = {None: "Algorithm 1", 0: "Algorithm 1", 1: "Ring Attention order", 2: "zigzag partition",
                  3: f"hybrid, {n_inner} devices per node"}[schedule]
    return {"workload": f"{name}: S={cfg.S} as {n} segments, Hq={cfg.Hq}, Hkv={cfg.Hkv}, causal={cfg.causal}, {sched_name}",
            "form": ("Update fused into the attention epilogue" if fused else
                     "tr_block_attn + tr_merge per step" + (", bf16 block_out" if block_dtype == tr.TR_BF16 else ", fp32 block_out")),
            "block_steps": full_steps + diag_steps, "ms": ms, "tflops": flops / (ms * 1e-3) / 1e12,
            "frac_mfma_peak": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}


def _blas_threads():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] or [1]))
    except Exception:
        return int(os.cpu_count() or 1)


def cpu_baseline(wl, budget_s=10.0):
    """The fp64 oracle on heads of the same block step, on this machine's host cores, for about budget_s seconds."""
    import oracle
    threads = _blas_threads()
    cfg = wl.CONFIGS["cfg2_block"]
    qb, kb, vb = wl.make_qkv_bits(cfg)
    f = wl.bf16_bits_to_f64
    heads, t_used = 0, 0.0
    while heads == 0 or t_used < budget_s:
        h = heads % cfg.Hq
        t0 = time.perf_counter()
        oracle.attention_block(f(qb[:, h:h + 1]), f(kb[:, h:h + 1]), f(vb[:, h:h + 1]), cfg.scale)
        t_used += time.perf_counter() - t0
        heads += 1
    flops = 4.0 * cfg.S * cfg.S * cfg.D * heads
    return {"value": flops / t_used / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"{heads} head-passes (heads taken cyclically out of {cfg.Hq}) of the 4096x4096 D=128 block step, "
                      f"fp64 numpy, {t_used:.1f} s"}


def oracle_timings(wl):
    """The oracle on the other workloads, each on a bounded sample (a few seconds): the small ring workload in full,
    a down-scaled merge-only workload, and sampled rows of one head of the two long causal rings, whose time for
    the whole workload is extrapolated by the ratio of (query, key) pairs."""
    import numpy as np
    import oracle
    f = wl.bf16_bits_to_f64
    res = {"cores": _blas_threads()}
    cfg = wl.CONFIGS["cfg1_small"]
    qb, kb, vb = wl.make_qkv_bits(cfg)
    t0 = time.perf_counter()
    reps = 0
    while reps == 0 or time.perf_counter() - t0 < 1.0:
        oracle.ring_attention(f(qb), f(kb), f(vb), cfg.n_chunks, cfg.causal, cfg.scale)
        reps += 1
    res["cfg1_ring_full"] = {"ms": (time.perf_counter() - t0) * 1e3 / reps, "what": "Algorithm 1 replayed by the oracle, whole workload"}
    mc = wl.CONFIGS["cfg4_merge"]
    S4 = 1024
    outs, lses = wl.make_merge_partials(mc, S=S4)
    t0 = time.perf_counter()
    oracle.merge_nary(outs, lses)
    t = time.perf_counter() - t0
    byts = 3 * mc.n_partials * mc.B * mc.H * S4 * (mc.D + 1) * 4      # what the eight pairwise Updates move
    res["cfg4_merge_scaled"] = {"ms": t * 1e3, "gbs": byts / t / 1e9, "what": f"8 partials of [1,32,{S4},128] (1/32 of the workload), n-ary definition"}
    for name in ("cfg3_ring", "cfg5_gqa"):
        c = wl.CONFIGS[name]
        rng = np.random.Generator(np.random.PCG64(c.seed + 7))
        kh = rng.standard_normal((c.S, c.D)) * c.std          # one K/V head drawn like the workload (timing only)
        vh = rng.standard_normal((c.S, c.D)) * c.std
        rows = wl.sample_rows(c.S, c.chunk, 48, seed=c.seed + 1)
        qh = rng.standard_normal((len(rows), c.D)) * c.std
        t0 = time.perf_counter()
        oracle.attention_rows(qh, rows, kh, vh, c.scale, True)
        t = time.perf_counter() - t0
        pairs = float(np.sum(rows + 1))
        total_pairs = c.B * c.Hq * (c.S * (c.S + 1) / 2.0)
        res[name + "_extrapolated"] = {"sample_ms": t * 1e3, "sample": f"{len(rows)} query rows of one head ({pairs:.3g} pairs)",
                                       "tflops": 4.0 * c.D * pairs / t / 1e12,
                                       "whole_workload_s_extrapolated": t * total_pairs / pairs}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-extras", action="store_true", help="skip the merge-only and ring workloads")
    ap.add_argument("--extras", default="", help="comma-separated names of the extras to run (default: all of them)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ramp", action="store_true", help="skip the untimed half second that brings the device out of its idle clock state")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (untimed) so that HBM-traffic counters of a "
                         "profiler run can be scaled by what they read for a copy of known size")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (no collectives, no sharding); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2412_20501_amd.build import ensure_built
    ensure_built()              # compiles unless the library on disk was built from exactly these sources
    import paper_2412_20501_amd as tr
    import workloads as wl
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    tr.raw_lib()   # fails loudly if libtokenring.so is missing
    print(f"bench.py: {tr.tr_version()} on {torch.cuda.get_device_name(0)}", file=sys.stderr)

    if args.calibration_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    r = bench_block_step(tr, wl, args.steps, args.warmup, 0.0 if args.no_ramp else 0.6)
    cfg = r["cfg"]
    value = r["flops"] / (r["ms_per_step"] * 1e-3) / 1e12
    line = {
        "metric": "block-attn TFLOP/s (one Algorithm-1 iteration: block attention + lse merge)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"], "ms_per_step_with_kernel_events": r["ms_per_step_events"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "cfg2 block step: B1 H32 Sq4096 x Sk4096 D128 bf16 N(0,1), non-causal, "
                               "bf16 block_out + fp32 block_lse merged into fp32 accumulators",
                   "seed": cfg.seed, "scale": cfg.scale, "library": tr.tr_version(),
                   "clock_ramp_s": 0.0 if args.no_ramp else 0.6},
        "roofline": {"bound": "mfma", "kernel": "block_attn_kernel<128,bf16 out>", "achieved": r["attn_tflops"],
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": r["attn_tflops"] / PEAK_BF16_TFLOPS,
                     "traffic": _traffic("block_attn_cfg2"), "ms_avg": r["attn_ms_avg"], "ms_median": r["attn_ms_median"],
                     "ms_min": r["attn_ms_min"], "flops_per_launch": r["flops"]},
        "merge_roofline": {"bound": "hbm", "kernel": "merge_kernel<bf16 block>", "achieved": r["merge_gbs"],
                           "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": r["merge_gbs"] / PEAK_HBM_GBS,
                           "traffic": _traffic("merge_cfg2"), "ms_avg": r["merge_ms_avg"], "ms_median": r["merge_ms_median"],
                           "ms_min": r["merge_ms_min"], "bytes_per_launch": r["merge_bytes"]},
        "parity": r["parity"],
    }
    if not args.no_extras:
        ex_steps = max(3, min(args.steps, 10))
        table = {
            "library_gemm_ceiling": lambda: bench_gemm_ceiling(),
            "step_fused": lambda: bench_step_fused(tr, wl, ex_steps, 2),
            "block_diag": lambda: bench_block(tr, wl, "cfg2_block_diag", ex_steps, 2, "cfg2 diagonal-causal block step"),
            "block_wide_scores": lambda: bench_block(tr, wl, "cfg2_block_wide", ex_steps, 2,
                                                     "cfg2 block step with Q, K ~ N(0, 3^2): scaled scores about 9 standard deviations wide"),
            "block_ramp_scores": lambda: bench_block(tr, wl, "cfg2_block_ramp", ex_steps, 2,
                                                     "cfg2 block step with scores rising 0.01 per key (+41 over the chunk)"),
            "merge_only": lambda: bench_merge_only(tr, wl, 3, 1),
            "ring_cfg1": lambda: bench_ring_small(tr, wl),
            "ring_cfg3": lambda: bench_ring(tr, wl, "cfg3_ring", ex_steps, 1, fused=True),
            "ring_cfg3_two_kernel": lambda: bench_ring(tr, wl, "cfg3_ring", ex_steps, 1, fused=False),
            "ring_cfg3_two_kernel_bf16_blocks": lambda: bench_ring(tr, wl, "cfg3_ring", ex_steps, 1, fused=False, block_dtype=tr.TR_BF16),
            "ring_cfg3_zigzag": lambda: bench_ring(tr, wl, "cfg3_ring", ex_steps, 1, fused=True, schedule=tr.TR_SCHED_ZIGZAG),
            "ring_cfg3_hybrid_2x4": lambda: bench_ring(tr, wl, "cfg3_ring", ex_steps, 1, fused=True, schedule=tr.TR_SCHED_HYBRID, n_inner=4),
            "ring_cfg5": lambda: bench_ring(tr, wl, "cfg5_gqa", 2, 1, fused=True),
            "ring_dit": lambda: bench_ring(tr, wl, "dit_ring", ex_steps, 1, fused=True),
        }
        chosen = [n for n in args.extras.split(",") if n] or list(table)
        unknown = [n for n in chosen if n not in table]
        if unknown:
            print(f"bench.py: unknown extras {unknown}; known: {list(table)}", file=sys.stderr)
            sys.exit(2)
        line["extras"] = {n: table[n]() for n in chosen}
        torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(wl)
        if not args.no_extras and not args.extras:
            line["extras"]["oracle_timings"] = oracle_timings(wl)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
