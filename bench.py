#!/usr/bin/env python3
"""Benchmark of the attention forward on one MI355X.

A step is one fa_fwd launch over one batch of synthetic input already resident in HBM.
Prints ONE JSON line: whole-job TFLOP/s on the headline workload -- C5, the long-context causal
configuration (B=1, H=32, N=131072, D=128, bf16), the largest of the benchmark's configurations and the
one the ">= 50% of MFMA peak on the causal long-sequence configurations" target is about -- with the
roofline figures of the kernel measured with HIP events on the launch stream, the output of the timed
launches checked against the CPU oracle (every element for C1/C2, the seeded sample of 64 rows per head
for C3-C5), the oracle timed on the host cores, and (unless --no-extra) the other configurations, each
with its own roofline entry.

FLOP convention (section 5.2.3 of the paper, times the batch): 4*B*H*Nq*Nk*D, halved when causal.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense fp16/bf16 MFMA peak
HBM_PEAK_GBS = 8000.0       # MI355X HBM3E peak
METRIC = "attention fwd TFLOP/s and % of MFMA fp16/bf16 peak (1 MI355X)"


def device_inputs_host_recipe(cfg, torch, np, I):
    """The seeded numpy recipe (exactly the tensors the parity tests check), copied to the GPU."""
    q, k, v = I.make_qkv(cfg)
    dev = torch.device("cuda:0")
    return tuple(torch.from_numpy(a.view(np.int16)).to(dev) for a in (q, k, v)), (q, k, v)


def device_inputs_on_gpu(cfg, torch):
    """Same distribution, drawn on the GPU from torch's seeded generator (for the large extras)."""
    dev = torch.device("cuda:0")
    tdt = torch.float16 if cfg.dtype == 0 else torch.bfloat16
    g = torch.Generator(device=dev)
    out = []
    for seed, n in zip(cfg.seeds, (cfg.Nq, cfg.Nk, cfg.Nk)):
        g.manual_seed(seed)
        t = torch.empty((cfg.B, cfg.H, n, cfg.D), dtype=tdt, device=dev)
        for b in range(cfg.B):   # per batch entry: bounds the fp32 temporary
            x = torch.randn((cfg.H, n, cfg.D), generator=g, device=dev, dtype=torch.float32)
            t[b] = (x * cfg.mult).to(tdt)
        out.append(t.view(torch.int16))
    return tuple(out)


MIN_WARM_S = 0.5   # the untimed warm-up lasts at least this long, so that the timed steps run at sustained clocks


def time_config(cfg, tensors, steps, warmup, torch, fa):
    """Warm up (`warmup` launches, and on until MIN_WARM_S seconds have passed: the warm-up is untimed, and a
    timed region that starts on a GPU still ramping its clocks reads 10% low), then time exactly `steps`
    launches.  Returns wall ms/step and the HIP-event mean ms/launch."""
    tq, tk, tv = tensors
    dev = tq.device
    to = torch.empty((cfg.B, cfg.H, cfg.Nq, cfg.D), dtype=torch.int16, device=dev)
    tl = torch.empty((cfg.B, cfg.H, cfg.Nq), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream

    def launch():
        fa.fa_fwd(tq, tk, tv, to, tl, cfg.B, cfg.H, cfg.Nq, cfg.Nk, cfg.D, cfg.scale, int(cfg.causal), cfg.dtype, sp)

    t_w = time.perf_counter()
    done = 0
    while done < warmup or time.perf_counter() - t_w < MIN_WARM_S:
        for _ in range(max(1, min(warmup, 50))):
            launch()
        done += max(1, min(warmup, 50))
        torch.cuda.synchronize()
    time_config.last_warmup_launches = done
    # HIP events on the stream the kernel is launched on: one pair around all the steps, and one event per chunk
    # of steps (at most 20 chunks) for the spread
    nchunk = min(20, steps)
    bounds = [steps * i // nchunk for i in range(nchunk + 1)]
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(nchunk + 1)]
    t0 = time.perf_counter()
    evs[0].record(stream)
    for c in range(nchunk):
        for _ in range(bounds[c + 1] - bounds[c]):
            launch()
        evs[c + 1].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall_ms = (t1 - t0) * 1e3 / steps
    event_ms = evs[0].elapsed_time(evs[-1]) / steps
    chunk_ms = sorted(evs[c].elapsed_time(evs[c + 1]) / (bounds[c + 1] - bounds[c]) for c in range(nchunk))
    time_config.last_spread = {"chunks": nchunk, "min_ms": round(chunk_ms[0], 5),
                               "median_ms": round(chunk_ms[len(chunk_ms) // 2], 5), "max_ms": round(chunk_ms[-1], 5)}
    return wall_ms, event_ms, (to, tl)


def time_decode(cfg, tensors, steps, warmup, torch, fa):
    """The decoding workload through fa_fwd_splitkv (workspace allocated once, outside the timed region).
    Returns the HIP-event mean ms per call (two kernels: partial attention + merge) and the plan."""
    tq, tk, tv = tensors
    dev = tq.device
    to = torch.empty((cfg.B, cfg.H, cfg.Nq, cfg.D), dtype=torch.int16, device=dev)
    tl = torch.empty((cfg.B, cfg.H, cfg.Nq), dtype=torch.float32, device=dev)
    plan = fa.fa_fwd_splitkv_plan(cfg.B, cfg.H, cfg.Nq, cfg.Nk, cfg.D, int(cfg.causal), cfg.dtype, 0)
    ws = torch.empty((plan.workspace_bytes + 3) // 4, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream

    def launch():
        fa.fa_fwd_splitkv(tq, tk, tv, to, tl, cfg.B, cfg.H, cfg.Nq, cfg.Nk, cfg.D, cfg.scale, int(cfg.causal),
                          cfg.dtype, 0, ws, plan.workspace_bytes, sp)

    for _ in range(warmup):
        launch()
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    ev0.record(stream)
    for _ in range(steps):
        launch()
    ev1.record(stream)
    torch.cuda.synchronize()
    return ev0.elapsed_time(ev1) / steps, plan


def mfma_ceiling(torch, fb, dtype, operands):
    """TFLOP/s of a kernel that issues nothing but matrix instructions (fa_mfma_probe of include/fa_bench.h), sustained for about 0.3 s:
    what the chip delivers under its power limit, to quote beside the nominal peak.  operands = 0: the same
    few-bit operands for every instruction; 1: pseudo-random operands that toggle from instruction to instruction."""
    scratch = torch.zeros(1, dtype=torch.float32, device="cuda:0")
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream
    iters = 200000
    for _ in range(2):
        flops = fb.fa_mfma_probe(dtype, operands, iters, scratch, sp)
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    reps = 4
    ev0.record(stream)
    for _ in range(reps):
        fb.fa_mfma_probe(dtype, operands, iters, scratch, sp)
    ev1.record(stream)
    torch.cuda.synchronize()
    return reps * flops / (ev0.elapsed_time(ev1) * 1e-3) / 1e12


def read_traffic(workload, stem="fa_fwd"):
    """HBM bytes per launch (per call for the entry points that enqueue several kernels).  NOT measured in this
    run: read from the committed summary of a separate rocprofv3 --pmc run (counters cannot be collected from
    inside the benchmark).  Returns (bytes or None, the file it came from or None)."""
    rel = os.path.join("profiles", f"{stem}_{workload}_hbm_traffic.txt")
    try:
        for line in open(os.path.join(ROOT, rel)):
            if line.startswith("traffic_bytes_per_launch:") or line.startswith("traffic_bytes_per_call:"):
                return float(line.split(":", 1)[1]), rel
    except OSError:
        pass
    return None, None


def traffic_fields(workload, stem="fa_fwd"):
    t, src = read_traffic(workload, stem)
    return {"traffic": t, "traffic_source": (src + " (separate rocprofv3 --pmc run, not this run)") if src else None}


def decode_entry(I, torch, fa, steps, warmup):
    """Appendix C's decoding shape through the split-KV entry point, priced against HBM: the algorithmic
    bytes of a call are K and V read once (Q, O, lse and the partial results are thousands of times smaller)."""
    c = I.DECODE
    tensors = device_inputs_on_gpu(c, torch)
    ms, plan = time_decode(c, tensors, steps, warmup, torch, fa)
    kv_bytes = 2.0 * c.B * c.H * c.Nk * c.D * 2
    gbs = kv_bytes / (ms * 1e-3) / 1e9
    return {"workload": c.describe(), "entry_point": "fa_fwd_splitkv", "nsplit": plan.nsplit,
            "grid": [plan.grid_x, plan.grid_y], "ms_per_call": round(ms, 5), "steps": steps,
            "inputs": "N(0,1) drawn on the GPU (torch generator, same seeds)",
            "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": round(gbs / HBM_PEAK_GBS, 4), **traffic_fields("splitkv_DEC"),
                         "kernel": ("fa_decode_kernel" if plan.streaming else "fa_fwd_kernel (wide, split-KV)")
                                   + " + fa_combine_kernel",
                         "bytes_per_call": kv_bytes}}


def sliding_entry(I, torch, fa, steps, warmup, c=None):
    """A causal sliding window through the descriptor-mask entry point, priced against the MFMA peak with the
    exact number of attending (query, key) pairs: 4*D flop each."""
    c = c or I.SLIDING
    tq, tk, tv = device_inputs_on_gpu(c, torch)
    dev = tq.device
    to = torch.empty((c.B, c.H, c.Nq, c.D), dtype=torch.int16, device=dev)
    tl = torch.empty((c.B, c.H, c.Nq), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream

    def launch():
        fa.fa_fwd_masked(tq, tk, tv, to, tl, c.B, c.H, c.Nq, c.Nk, c.D, c.scale, c.window - 1, 0, 0, None, c.dtype, sp)

    for _ in range(warmup):
        launch()
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    ev0.record(stream)
    for _ in range(steps):
        launch()
    ev1.record(stream)
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / steps
    tf = c.flops() / (ms * 1e-3) / 1e12
    return {"workload": c.describe(), "entry_point": "fa_fwd_masked", "ms_per_launch": round(ms, 4), "steps": steps,
            "inputs": "N(0,1) drawn on the GPU (torch generator, same seeds)",
            "flop_convention": "4*D per attending (query, key) pair, counted exactly",
            "roofline": {"bound": "mfma", "achieved": round(tf, 2), "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(tf / MFMA_PEAK_TFLOPS, 4), **traffic_fields("masked_" + c.name),
                         "kernel": "fa_fwd_kernel (wide, descriptor mask)", "flops_per_launch": c.flops()}}


def chunked_entry(I, torch, fa, steps, warmup):
    """Chunked prefill (a block of new tokens against a long cache) through the split-KV entry point, priced
    against the MFMA peak with the exact number of attending pairs (the chunk's own triangle is missing from the
    rectangle)."""
    c = I.CHUNKED
    tensors = device_inputs_on_gpu(c, torch)
    ms, plan = time_decode(c, tensors, steps, warmup, torch, fa)
    fl = 4.0 * c.D * c.visible_pairs()
    tf = fl / (ms * 1e-3) / 1e12
    kv_bytes = 2.0 * c.B * c.H * c.Nk * c.D * 2
    return {"workload": c.describe(), "entry_point": "fa_fwd_splitkv", "nsplit": plan.nsplit,
            "grid": [plan.grid_x, plan.grid_y], "ms_per_call": round(ms, 5), "steps": steps,
            "inputs": "N(0,1) drawn on the GPU (torch generator, same seeds)",
            "flop_convention": "4*D per attending (query, key) pair, counted exactly",
            "kv_gb_per_s": round(kv_bytes / (ms * 1e-3) / 1e9, 1),
            "roofline": {"bound": "mfma", "achieved": round(tf, 2), "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(tf / MFMA_PEAK_TFLOPS, 4), **traffic_fields("splitkv_CHUNK"),
                         "kernel": "fa_fwd_wide64_kernel (split-KV) + fa_combine_kernel", "flops_per_call": fl,
                         "note": "K and V are read once (512 MiB): at this arithmetic intensity (about 500 flop per "
                                 "byte) the HBM roofline allows 4 PFLOP/s, so the matrix peak is the bound"}}


def projection_entry(I, torch, fa, steps, warmup, overlap_demo=True):
    """Attention + output projection per block of rows (fa_attn_linear), priced against the MFMA peak:
    attention flop (causal convention) + 2 * tokens * (H*D) * N for the projection."""
    import math
    c = I.PROJECTION
    n_out, rpb = I.PROJECTION_N, I.PROJECTION_ROWS_PER_BLOCK
    tq, tk, tv = device_inputs_on_gpu(c, torch)
    dev = tq.device
    tdt = torch.float16 if c.dtype == 0 else torch.bfloat16
    g = torch.Generator(device=dev)
    g.manual_seed(c.seeds[2] + 1)
    tw = (torch.randn((c.H * c.D, n_out), generator=g, device=dev, dtype=torch.float32)
          / math.sqrt(c.H * c.D)).to(tdt).view(torch.int16)
    to = torch.empty((c.B, c.H, c.Nq, c.D), dtype=torch.int16, device=dev)
    tl = torch.empty((c.B, c.H, c.Nq), dtype=torch.float32, device=dev)
    ty = torch.empty((c.B, c.Nq, n_out), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream

    def launch():
        fa.fa_attn_linear(tq, tk, tv, tw, to, tl, ty, c.B, c.H, c.Nq, c.Nk, c.D, n_out, c.scale, int(c.causal), c.dtype,
                          rpb, sp)

    for _ in range(warmup):
        launch()
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    ev0.record(stream)
    for _ in range(steps):
        launch()
    ev1.record(stream)
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / steps
    fl_attn = c.flops()
    fl_proj = 2.0 * c.B * c.Nq * c.H * c.D * n_out
    tf = (fl_attn + fl_proj) / (ms * 1e-3) / 1e12

    # What the block-by-block form is for (section 4.2): the exchange of block i's partial sums runs while block
    # i + 1 is computed.  On one GPU a stand-in takes the exchange's place: COPIES device copies of the block's
    # rows of y on a second stream (default priority), behind an event recorded after the block's kernels.
    COPIES = 4
    ty2 = torch.empty_like(ty)
    side = torch.cuda.Stream(device=dev)
    blocks, r = [], 0
    while r < c.Nq:
        n = min(rpb // 2 if r == 0 else rpb, c.Nq - r)
        blocks.append((r, n))
        r += n

    def exchange(r, n):
        for _ in range(COPIES):
            ty2[:, r:r + n].copy_(ty[:, r:r + n])

    def pipeline(overlap, compute=True, comm=True):
        for r, n in blocks:
            if compute:
                fa.fa_attn_linear_block(tq, tk, tv, tw, to, tl, ty, c.B, c.H, c.Nq, c.Nk, c.D, n_out, c.scale,
                                        int(c.causal), c.dtype, r, n, sp)
            if comm:
                if overlap:
                    ev = torch.cuda.Event()
                    ev.record(stream)
                    side.wait_event(ev)
                    with torch.cuda.stream(side):
                        exchange(r, n)
                else:
                    exchange(r, n)
        if overlap:
            stream.wait_stream(side)

    def time_pipeline(**kw):
        for _ in range(max(2, warmup // 2)):
            pipeline(**kw)
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        reps = max(5, steps // 4)
        e0.record(stream)
        for _ in range(reps):
            pipeline(**kw)
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    overlap_entry = None
    if overlap_demo:
        t_compute = time_pipeline(overlap=False, comm=False)
        t_comm = time_pipeline(overlap=False, compute=False)
        t_serial = time_pipeline(overlap=False)
        t_overlap = time_pipeline(overlap=True)
        overlap_entry = {"stand_in": f"{COPIES} device copies of each block's rows of y on a second stream",
                         "ms_compute_only": round(t_compute, 4), "ms_exchange_only": round(t_comm, 4),
                         "ms_one_stream": round(t_serial, 4), "ms_two_streams": round(t_overlap, 4),
                         "exchange_hidden_frac": round((t_serial - t_overlap) / t_comm, 3)}
    return {"workload": c.describe() + f" + projection {c.H * c.D}x{n_out}, blocks of {rpb} rows (first one half)",
            "overlap_with_exchange_stand_in": overlap_entry,
            "entry_point": "fa_attn_linear", "ms_per_call": round(ms, 4), "steps": steps,
            "inputs": "N(0,1) drawn on the GPU (torch generator, same seeds); w ~ N(0,1)/sqrt(H*D)",
            "roofline": {"bound": "mfma", "achieved": round(tf, 2), "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(tf / MFMA_PEAK_TFLOPS, 4), **traffic_fields("LIN", "fa_attn_linear"),
                         "kernel": "fa_fwd_kernel + fa_linear_kernel, per block",
                         "flops_per_call": fl_attn + fl_proj, "flops_attention": fl_attn, "flops_projection": fl_proj}}


def rotating_entry(cfg, torch, fa, copies, steps, warmup):
    """The same workload with `copies` separate sets of Q, K, V, O taken in turn, so that a launch finds none of
    its tensors in the 256 MiB Infinity Cache (copies x 64 MiB for C2): the figure for inputs that really come
    from HBM, to quote beside the headline, whose single set stays cache-resident."""
    sets = []
    for _ in range(copies):
        tq, tk, tv = device_inputs_on_gpu(cfg, torch)
        to = torch.empty((cfg.B, cfg.H, cfg.Nq, cfg.D), dtype=torch.int16, device=tq.device)
        tl = torch.empty((cfg.B, cfg.H, cfg.Nq), dtype=torch.float32, device=tq.device)
        sets.append((tq, tk, tv, to, tl))
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream

    def launch(i):
        tq, tk, tv, to, tl = sets[i % copies]
        fa.fa_fwd(tq, tk, tv, to, tl, cfg.B, cfg.H, cfg.Nq, cfg.Nk, cfg.D, cfg.scale, int(cfg.causal), cfg.dtype, sp)

    for i in range(warmup):
        launch(i)
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    ev0.record(stream)
    for i in range(steps):
        launch(i)
    ev1.record(stream)
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / steps
    tf = cfg.flops() / (ms * 1e-3) / 1e12
    bytes_per_launch = 4.0 * cfg.B * cfg.H * cfg.Nq * cfg.D * 2 + 4.0 * cfg.B * cfg.H * cfg.Nq
    return {"workload": cfg.describe() + f", {copies} sets of tensors in rotation", "ms_per_launch": round(ms, 5),
            "tflops": round(tf, 2), "pct_of_mfma_peak": round(100.0 * tf / MFMA_PEAK_TFLOPS, 2), "steps": steps,
            "hbm_gb_per_s_algorithmic": round(bytes_per_launch / (ms * 1e-3) / 1e9, 1),
            "inputs": "N(0,1) drawn on the GPU (torch generator, same seeds)"}


def cpu_decode_entry(I, np):
    """The host-side decoding attention of the cooperative strategy (fa_cpu_decode) on one GPU's share of the
    decoding workload's heads, timed on the machine's host cores; bytes = K and V read once."""
    from paper_2410_16663_amd import cpu_binding as fc
    from paper_2410_16663_amd import bench_binding as fb
    c = I.DECODE
    B, H = 1, 32    # 512 MiB of K and V: far beyond the host's caches
    q = I.normal_bits((B, H, 1, c.D), c.seeds[0], c.dtype)
    # one head's worth of N(0,1) values, copied to every head (the timing does not depend on the values, and
    # drawing 2^28 normals on the host would take longer than everything else in this file)
    k = np.ascontiguousarray(np.broadcast_to(I.normal_bits((1, 1, c.Nk, c.D), c.seeds[1], c.dtype), (B, H, c.Nk, c.D)))
    v = np.ascontiguousarray(np.broadcast_to(I.normal_bits((1, 1, c.Nk, c.D), c.seeds[2], c.dtype), (B, H, c.Nk, c.D)))
    o = np.empty((B, H, 1, c.D), dtype=np.uint16)
    lse = np.empty((B, H, 1), dtype=np.float32)
    fc.fa_cpu_decode(q, k, v, o, lse, B, H, c.Nk, c.D, c.scale, c.dtype, 0)     # warm-up
    reps = 10
    t0 = time.perf_counter()
    for _ in range(reps):
        fc.fa_cpu_decode(q, k, v, o, lse, B, H, c.Nk, c.D, c.scale, c.dtype, 0)
    ms = (time.perf_counter() - t0) * 1e3 / reps
    kv_bytes = 2.0 * B * H * c.Nk * c.D * 2
    gbs = kv_bytes / (ms * 1e-3) / 1e9
    # the yardstick: the same threads adding up the same K and V buffers, nothing else
    fb.fa_cpu_stream_read(k, k.nbytes, 0, 1)
    stream = 0.5 * (fb.fa_cpu_stream_read(k, k.nbytes, 0, 5)[0] + fb.fa_cpu_stream_read(v, v.nbytes, 0, 5)[0])
    return {"workload": f"B={B} H={H} Nq=1 Nk={c.Nk} D={c.D} bf16 (host memory)", "entry_point": "fa_cpu_decode",
            "ms_per_call": round(ms, 4), "gb_per_s": round(gbs, 2),
            "threads": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), "avx512": fc.fa_cpu_has_avx512(),
            "bytes_per_call": kv_bytes,
            "roofline": {"bound": "host memory", "achieved": round(gbs, 1), "peak": round(stream, 1), "unit": "GB/s",
                         "frac": round(gbs / stream, 4), "traffic": None,
                         "peak_is": "fa_cpu_stream_read (include/fa_bench.h) over the same buffers on the same threads (measured, "
                                    "not a published figure)"}}


FULL_ORACLE = ("C1", "C2")    # checked element by element; the others on the seeded sample of 64 rows per (b, h)


def oracle_leg(cfg, host, outputs, np, I, time_it):
    """The timed launches' output against the fp64 oracle -- every element for C1/C2, the seeded stratified sample
    of 64 rows per (batch, head) (inputs.sample_rows) for C3-C5, whose full oracle would take hours -- and, with
    time_it, the oracle itself timed on the host cores over the same rows (whole passes until about 20
    core-seconds are spent).  Returns (parity dict, cpu_baseline dict or None)."""
    import oracle
    q, k, v = host
    nthreads = min(oracle.num_threads(), os.cpu_count() or 1)
    full = cfg.name in FULL_ORACLE
    rows = None if full else I.sample_rows(cfg)
    nrows = cfg.B * cfg.H * cfg.Nq if full else int(rows.size)
    if full:
        pairs = cfg.visible_pairs()
    else:
        i = rows % cfg.Nq
        pairs = int(np.clip(i + (cfg.Nk - cfg.Nq) + 1, 0, cfg.Nk).sum()) if cfg.causal else nrows * cfg.Nk
    t0 = time.perf_counter()
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, cfg.scale, cfg.causal, cfg.dtype, rows=rows, nthreads=nthreads)
    passes, dt = 1, time.perf_counter() - t0
    cpu = None
    if time_it:
        while dt * nthreads < 20.0 and passes < 8:
            oracle.attention_fwd(q, k, v, cfg.scale, cfg.causal, cfg.dtype, rows=rows, nthreads=nthreads)
            passes += 1
            dt = time.perf_counter() - t0
        # convention flop of the rows the oracle did: 4*D per visible (query, key) pair
        fl = 4.0 * cfg.D * pairs * passes
        cpu = {"value": round(fl / dt / 1e12, 6), "unit": "TFLOP/s", "cores": nthreads, "kind": "oracle",
               "seconds": round(dt, 3),
               "sample": (f"all {nrows} query rows of {cfg.name}" if full else
                          f"{nrows} of the {cfg.B * cfg.H * cfg.Nq} query rows of {cfg.name} (the seeded stratified "
                          f"sample of 64 rows per head, {pairs:.3e} visible pairs)") + f", {passes} pass(es), fp64",
               "flop_counted": "4*D per visible (query, key) pair of the rows computed",
               "extrapolated_seconds_for_the_whole_workload": round(dt / passes * cfg.visible_pairs() / pairs, 1)}
    to, tl = outputs
    o_all = to.cpu().numpy().view(np.uint16)
    lse_all = tl.cpu().numpy().astype(np.float64)
    if full:
        o, lse = I.bits_to_f64(o_all, cfg.dtype), lse_all
    else:
        o, lse = I.bits_to_f64(o_all.reshape(-1, cfg.D)[rows], cfg.dtype), lse_all.reshape(-1)[rows]
    err = np.abs(o - o_ref)
    o_ref_rounded = I.bits_to_f64(I.f32_to_bits(o_ref.astype(np.float32), cfg.dtype), cfg.dtype)
    worst = np.unravel_index(int(np.argmax(err)), err.shape)
    fin = np.isfinite(lse_ref)
    parity = {"against": "fp64 oracle, " + ("every element of the timed output" if full else
                                           f"{nrows} sampled rows of the timed output (64 per head, stratified, "
                                           "seeded; the other rows are not oracle-checked)"),
              "o_max_abs": float(err.max()), "o_mean_abs": float(err.mean()),
              "lse_max_abs": float(np.abs(lse[fin] - lse_ref[fin]).max()),
              "o_max_abs_vs_oracle_rounded_to_dtype": float(np.abs(o - o_ref_rounded).max()),
              "elements_over_1e-2": int((err > 1e-2).sum()), "elements_checked": int(err.size),
              "worst_element": [int(x) for x in worst] if full else
                               {"flat_row": int(rows[worst[0]]), "d": int(worst[1])},
              "all_lse_finite": bool(np.isfinite(lse_all).all()),
              "tolerance": {"o_max_abs": 1e-2, "o_mean_abs": 1e-3, "lse_abs": 1e-3},
              "pass": bool(err.max() <= 1e-2 and err.mean() <= 1e-3 and np.abs(lse[fin] - lse_ref[fin]).max() <= 1e-3)}
    return parity, cpu


KERNEL_OF_MODE = {0: "fa_fwd_kernel (split)", 1: "fa_fwd_kernel (wide)", 2: "fa_fwd_kernel (wide, folded rows)",
                  3: "fa_decode_kernel (streaming decode)", 4: "fa_fwd_wide64_kernel (64-row waves, pipelined loop)"}


def roofline_entry(cfg, event_ms, plan):
    flops = cfg.flops()
    achieved = flops / (event_ms * 1e-3) / 1e12
    return {"bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(achieved / MFMA_PEAK_TFLOPS, 4), **traffic_fields(cfg.name),
            "kernel": KERNEL_OF_MODE[plan.mode], "avg_launch_ms": round(event_ms, 5),
            "flops_per_launch": flops,
            "timing": "HIP events on the launch stream around the timed steps"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed launches (default: 20 for C5, more for the shorter ones)")
    ap.add_argument("--warmup", type=int, default=None,
                    help="untimed launches before (default: a quarter of --steps); the warm-up also lasts at least "
                         "half a second whatever this says")
    ap.add_argument("--workload", default="C5", help="headline workload (C1..C5)")
    ap.add_argument("--sliding-only", action="store_true",
                    help="time only the sliding-window workload through fa_fwd_masked (for profiling runs)")
    ap.add_argument("--projection-only", action="store_true",
                    help="time only the attention + output projection workload (for profiling runs)")
    ap.add_argument("--overlap-demo", action="store_true",
                    help="with --projection-only: also time the two-stream pipeline with the exchange stand-in")
    ap.add_argument("--no-linear-overlap", action="store_true",
                    help="fa_attn_linear keeps its projections on the caller's stream (for comparison runs)")
    ap.add_argument("--chunked-only", action="store_true",
                    help="time only the chunked-prefill workload through fa_fwd_splitkv (for profiling runs)")
    ap.add_argument("--sliding64-only", action="store_true",
                    help="time only the sliding-window workload at head dimension 64 (for profiling runs)")
    ap.add_argument("--decode-only", action="store_true",
                    help="time only the decoding workload through fa_fwd_splitkv (for profiling runs)")
    ap.add_argument("--fwd-mode", default=None, choices=["split", "wide", "fold", "wide64"],
                    help="force fa_fwd's work decomposition (fa_set_option; for profiling and tuning runs)")
    ap.add_argument("--no-extra", action="store_true", help="skip the other configurations and workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle (baseline and parity)")
    ap.add_argument("--gpu-inputs", action="store_true",
                    help="draw the headline workload's inputs on the GPU (implies --no-cpu); for profiling runs")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="also launch a plain device copy of this many MiB (a known-size reference "
                         "for the HBM byte counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.steps is None:
        args.steps = {"C1": 20000, "C2": 20000, "C3": 200, "C4": 600, "C5": 20}.get(args.workload, 50)
        if args.decode_only:
            args.steps = 2000
        if args.sliding_only or args.projection_only or args.sliding64_only or args.chunked_only:
            args.steps = 200
    if args.warmup is None:
        args.warmup = max(1, args.steps // 4)
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2410_16663_amd import binding as fa
    from paper_2410_16663_amd import bench_binding as fb
    from paper_2410_16663_amd import inputs as I

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    fa.load()   # fails loudly if libfa.so is missing; there is no fallback
    torch.cuda.set_device(0)

    if args.fwd_mode:
        fa.fa_set_option(fa.FA_OPT_FWD_MODE, {"split": fa.FA_MODE_SPLIT, "wide": fa.FA_MODE_WIDE,
                                              "fold": fa.FA_MODE_WIDE_FOLD, "wide64": fa.FA_MODE_WIDE64}[args.fwd_mode])
    if args.no_linear_overlap:
        fa.fa_set_option(fa.FA_OPT_LINEAR_OVERLAP, 0)
    cfg = I.CONFIGS[args.workload]
    if args.copy_calibration > 0:
        n = args.copy_calibration * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.sliding_only:
        print(json.dumps({"sliding": sliding_entry(I, torch, fa, args.steps, args.warmup)}), flush=True)
        return
    if args.sliding64_only:
        print(json.dumps({"sliding64": sliding_entry(I, torch, fa, args.steps, args.warmup, I.SLIDING64)}), flush=True)
        return
    if args.chunked_only:
        print(json.dumps({"chunked": chunked_entry(I, torch, fa, args.steps, args.warmup)}), flush=True)
        return
    if args.projection_only:
        print(json.dumps({"projection": projection_entry(I, torch, fa, args.steps, args.warmup, args.overlap_demo)}),
              flush=True)
        return
    if args.decode_only:
        print(json.dumps({"decode": decode_entry(I, torch, fa, args.steps, args.warmup)}), flush=True)
        return
    if args.gpu_inputs:
        args.no_cpu = True
        tensors, host = device_inputs_on_gpu(cfg, torch), None
    else:
        tensors, host = device_inputs_host_recipe(cfg, torch, np, I)
    wall_ms, event_ms, outputs = time_config(cfg, tensors, args.steps, args.warmup, torch, fa)
    spread = time_config.last_spread
    warm_launches = time_config.last_warmup_launches
    ceiling = mfma_ceiling(torch, fb, cfg.dtype, 0)
    ceiling_random = mfma_ceiling(torch, fb, cfg.dtype, 1)
    flops = cfg.flops()
    plan = fa.fa_fwd_plan(cfg.B, cfg.H, cfg.Nq, cfg.Nk, cfg.D, int(cfg.causal), cfg.dtype)
    value = flops / (wall_ms * 1e-3) / 1e12
    tensor_mib = 4 * cfg.B * cfg.H * cfg.Nq * cfg.D * 2 / 2 ** 20

    out = {
        "metric": METRIC, "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(wall_ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if cfg.dtype == 0 else "bf16", "data": "synthetic",
        "pct_of_mfma_peak": round(100.0 * value / MFMA_PEAK_TFLOPS, 2),
        "mfma_only_ceiling_tflops": round(ceiling, 1), "pct_of_mfma_only_ceiling": round(100.0 * value / ceiling, 2),
        "mfma_only_ceiling_random_operands_tflops": round(ceiling_random, 1),
        "pct_of_mfma_only_ceiling_random_operands": round(100.0 * value / ceiling_random, 2),
        "launch_time_spread": spread, "warmup_launches_actually_run": warm_launches,
        "config": {"workload": cfg.describe(), "flop_convention": "4*B*H*Nq*Nk*D, halved when causal",
                   "flops_exact_visible_pairs": 4.0 * cfg.D * cfg.visible_pairs(),
                   "accumulate": "fp32",
                   "inputs": ("N(0,1) drawn on the GPU (torch generator)" if host is None else
                              "N(0,1) numpy PCG64 seeds %s" % (cfg.seeds,)) + ", resident in HBM",
                   "note": f"Q,K,V,O of this workload are {tensor_mib:.0f} MiB"
                           + (" and fit in the 256 MiB Infinity Cache" if tensor_mib <= 256 else "")},
        "roofline": roofline_entry(cfg, event_ms, plan),
    }

    if not args.no_cpu:
        out["parity"], out["cpu_baseline"] = oracle_leg(cfg, host, outputs, np, I, True)

    if not args.no_extra:
        extra = {}
        del outputs
        if cfg.name == "C2":
            extra["C2_from_hbm"] = rotating_entry(cfg, torch, fa, 8, 8000, 2000)
        for name in ("C3", "C2", "C4", "C5"):
            if name == cfg.name:
                continue
            c = I.CONFIGS[name]
            del tensors
            torch.cuda.empty_cache()
            # C2 and C3 (the other causal D = 128 configurations): the seeded host recipe, so that their outputs can
            # be checked against the oracle too; C4 / C5 as extras: drawn on the GPU, timing only
            check = name in ("C2", "C3") and not args.no_cpu
            if check:
                tensors, h = device_inputs_host_recipe(c, torch, np, I)
            else:
                tensors, h = device_inputs_on_gpu(c, torch), None
            steps = {"C2": 20000, "C3": 100, "C4": 300, "C5": 5}[name]   # 0.3-1 s each
            w_ms, e_ms, outs = time_config(c, tensors, steps, max(1, steps // 10), torch, fa)
            pl = fa.fa_fwd_plan(c.B, c.H, c.Nq, c.Nk, c.D, int(c.causal), c.dtype)
            extra[name] = {"workload": c.describe(), "ms_per_launch": round(e_ms, 5),
                           "tflops": round(c.flops() / (e_ms * 1e-3) / 1e12, 2), "steps": steps,
                           "inputs": "N(0,1) numpy PCG64 seeds %s" % (c.seeds,) if check
                                     else "N(0,1) drawn on the GPU (torch generator, same seeds)",
                           "roofline": roofline_entry(c, e_ms, pl)}
            if check:
                extra[name]["parity"], _ = oracle_leg(c, h, outs, np, I, False)
            del outs, h
        del tensors
        torch.cuda.empty_cache()
        extra["DEC"] = decode_entry(I, torch, fa, 500, 50)
        torch.cuda.empty_cache()
        extra["SWA"] = sliding_entry(I, torch, fa, 60, 6)
        torch.cuda.empty_cache()
        extra["SWA64"] = sliding_entry(I, torch, fa, 60, 6, I.SLIDING64)
        torch.cuda.empty_cache()
        extra["CHUNK"] = chunked_entry(I, torch, fa, 300, 30)
        torch.cuda.empty_cache()
        extra["LIN"] = projection_entry(I, torch, fa, 100, 10)
        extra["CPU_DEC"] = cpu_decode_entry(I, np)
        out["other_workloads"] = extra

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
