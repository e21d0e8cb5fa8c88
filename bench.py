#!/usr/bin/env python3
"""Benchmark of the Flash-LoRA-Attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One step = one lra_attn_decode call (key-streaming kernel + split merge/epilogue)
on the Llama-3-8B-shaped 4-agent decode workload: n = 8192 cached tokens, 32 q /
8 kv heads, d = 128, r = 16, bf16.  Inputs are resident in HBM before the timed
region.  The working set (34 MB) would fit the 256 MB memory-side cache, so the
timed steps cycle through enough distinct copies of (K_base, V_base, L) that
every step streams its cache from HBM ("cold"); the same-buffer ("hot") figure
is reported next to it.  value = algorithmic bytes / step time.

The JSON line also carries
  roofline      the key-streaming kernel alone (no merge), HIP events on its stream
                around the same number of back-to-back launches,
  prefill       the causal prefill workload (2048 new tokens after 16384), TFLOP/s,
  rotary_key_prefill  the prefill workload with the rotary key side (key_rope_theta),
  cache_append  the producer of the caches (lra_cache_append) at the Llama-3-8B projection shape,
  cpu_baseline  the fp64 oracle timed on this machine's host cores.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published
COLD_BYTES = 600e6             # cycle through more than twice the 256 MB memory-side cache


def _hip():
    lib = ctypes.CDLL("libamdhip64.so")
    lib.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    lib.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    lib.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    lib.hipEventSynchronize.argtypes = [ctypes.c_void_p]
    lib.hipEventDestroy.argtypes = [ctypes.c_void_p]
    return lib


MIN_KERNEL_LAUNCHES = 200     # launches between one pair of events when a kernel is timed alone
MIN_TIMED_SECONDS = 0.02      # a timed region is repeated until it is at least this long


def graph_seconds(torch, launch, n, min_seconds=MIN_TIMED_SECONDS, max_replays=2000):
    """Seconds per launch of `launch(i, stream)`, i = 0..n-1, enqueued back to back: the n calls are
    captured into a HIP graph (so that no Python or ctypes time sits between two launches; a decode
    step is shorter than that overhead) and the graph is replayed between two HIP events on the
    stream it runs on, as often as it takes to fill min_seconds.  Returns (seconds per launch,
    launches timed).  A HIP event pair costs about 6 us here, which is why events bracket whole
    replays and never a single launch."""
    hip = _hip()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for i in range(min(n, 3)):
            launch(i, side)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for i in range(n):
            launch(i, side)
    graph.replay()
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream().cuda_stream or None
    e0, e1 = ctypes.c_void_p(), ctypes.c_void_p()
    assert hip.hipEventCreate(ctypes.byref(e0)) == 0 and hip.hipEventCreate(ctypes.byref(e1)) == 0
    ms = ctypes.c_float()
    replays, total, done = 1, 0.0, 0
    try:
        while True:
            assert hip.hipEventRecord(e0, stream) == 0
            for _ in range(replays):
                graph.replay()
            assert hip.hipEventRecord(e1, stream) == 0
            hip.hipEventSynchronize(e1)
            assert hip.hipEventElapsedTime(ctypes.byref(ms), e0, e1) == 0
            total, done = ms.value * 1e-3, replays
            if total >= min_seconds or replays >= max_replays:
                break
            replays = min(max_replays, max(replays * 2, int(replays * min_seconds / max(total, 1e-6)) + 1))
    finally:
        hip.hipEventDestroy(e0)
        hip.hipEventDestroy(e1)
        del graph
    return total / (done * n), done * n


def kernel_seconds(lra, torch, launch, n=MIN_KERNEL_LAUNCHES):
    """Average duration of the library's dominant kernel: at least MIN_KERNEL_LAUNCHES back-to-back
    launches of that kernel alone (lra_set_profile_mode(1): the call enqueues nothing else), timed by
    graph_seconds.  The figure includes the dispatch gap between consecutive launches."""
    n = max(n, MIN_KERNEL_LAUNCHES)
    old = lra.lra_set_profile_mode(1)
    try:
        sec, _ = graph_seconds(torch, launch, n)
    finally:
        lra.lra_set_profile_mode(old)
    return sec


def machine_ceilings(torch, lra):
    """What this GPU gives a plain streaming read (1.5 GB, far beyond the memory-side cache) and a
    register-resident bf16 MFMA loop (about half a second of sustained matrix work, so the clock settles
    where it does under such load): the library's two probe kernels, HIP events on their stream."""
    dev = torch.device("cuda:0")
    hip = _hip()
    stream = torch.cuda.current_stream().cuda_stream or None
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    e0, e1 = ctypes.c_void_p(), ctypes.c_void_p()
    assert hip.hipEventCreate(ctypes.byref(e0)) == 0 and hip.hipEventCreate(ctypes.byref(e1)) == 0

    def timed(launch, n):
        launch()
        torch.cuda.synchronize()
        assert hip.hipEventRecord(e0, stream) == 0
        for _ in range(n):
            launch()
        assert hip.hipEventRecord(e1, stream) == 0
        hip.hipEventSynchronize(e1)
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), e0, e1) == 0
        return ms.value * 1e-3 / n

    buf = torch.empty(1536 << 20, dtype=torch.uint8, device=dev)
    buf.fill_(1)
    read_s = timed(lambda: lra.lra_probe_stream_read(buf, sink), 20)
    hbm = buf.numel() / read_s / 1e9
    del buf
    flops = []
    mfma_s = timed(lambda: flops.append(lra.lra_probe_mfma_bf16(200000, sink)), 20)
    mfma_rand_s = timed(lambda: lra.lra_probe_mfma_bf16(200000, sink, random_operands=True), 20)
    hip.hipEventDestroy(e0)
    hip.hipEventDestroy(e1)
    return {"hbm_stream_read_GBps": round(hbm, 1), "hbm_frac_of_peak": round(hbm / HBM_PEAK_GBS, 4),
            "mfma_bf16_TFLOPs": round(flops[-1] / mfma_s / 1e12, 1),
            "mfma_frac_of_peak": round(flops[-1] / mfma_s / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
            "mfma_bf16_random_operands_TFLOPs": round(flops[-1] / mfma_rand_s / 1e12, 1),
            "note": "lra_probe_stream_read over 1.5 GB; lra_probe_mfma_bf16 with operands in registers, two smooth values "
                    "throughout and four pseudo-random registers in rotation; measured in this run"}


def stream_read_at_size(torch, lra, nbytes):
    """What the plain streaming-read probe reaches on a buffer of the workload's own size, launch
    for launch, taken in turn from enough distinct buffers that every launch reads from HBM: the
    ceiling a call that moves this many bytes can be held against (launch, ramp-up and drain
    included), unlike the 1.5 GB figure."""
    dev = torch.device("cuda:0")
    nbytes = (int(nbytes) + 255) // 256 * 256
    k = int(math.ceil(COLD_BYTES / nbytes)) + 1
    pool = torch.empty(k * nbytes, dtype=torch.uint8, device=dev)
    pool.fill_(1)
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    bufs = [pool[i * nbytes:(i + 1) * nbytes] for i in range(k)]
    sec, _ = graph_seconds(torch, lambda i, st: lra.lra_probe_stream_read(bufs[i % k], sink, st), max(MIN_KERNEL_LAUNCHES, 4 * k))
    del bufs, pool
    return sec


def _load_traffic(name):
    """HBM bytes per launch of the named kernel from the committed rocprofv3 --pmc summary (None if there
    is none), and whether that summary was taken on kernel sources other than the ones in this tree
    (profiles/traffic.json records the fingerprint of the sources it was measured on)."""
    from paper_2602_01053_amd.build import source_fingerprint
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return None, None
    return rec.get(name), rec.get("source_fingerprint") != source_fingerprint()


def _traffic_fields(roof, name, seconds):
    """Adds the rocprofv3-measured HBM bytes per launch, the rate they give over the kernel time
    measured in this run, and the staleness flag to a roofline object."""
    traffic, stale = _load_traffic(name)
    roof["traffic"] = traffic
    if traffic is not None:
        roof["traffic_GBps"] = round(traffic / seconds / 1e9, 1)
        roof["traffic_measured_on_other_sources"] = bool(stale)
    return roof


def bench_decode(args, torch, lra, workloads, index=2, steps=None, warmup=None, value_only=False, kernel_only=False):
    """Times one decode configuration.  Caches smaller than COLD_BYTES are rotated over
    enough copies that every step streams from HBM.  value_only passes b_k = NULL (keys
    fully shared, LoRA on the value side only: the paper's main setting)."""
    from paper_2602_01053_amd.runner import DeviceWorkload
    steps = steps or args.steps
    warmup = warmup or args.warmup
    dev = torch.device("cuda:0")
    w = workloads.config(index)
    alg_bytes = w.algorithmic_bytes()
    cache_bytes = (2 * w.k_base.numel() + w.l.numel()) * w.k_base.element_size()
    n_copies = 1 if cache_bytes >= COLD_BYTES else int(math.ceil(COLD_BYTES / cache_bytes)) + 1
    base = DeviceWorkload(w, dev)
    base.alloc_workspace()
    if value_only:
        base.b_k = None
    copies = [base]
    for _ in range(n_copies - 1):
        c = DeviceWorkload.__new__(DeviceWorkload)
        c.__dict__.update(base.__dict__)
        c.k_base, c.v_base, c.l = base.k_base.clone(), base.v_base.clone(), base.l.clone()
        c.cache = lra.make_cache(c.k_base, c.v_base, c.l, c.seq_lens, max(w.seq_lens), c.block_table)
        copies.append(c)

    def run(n_steps, cold):
        for i in range(n_steps):
            copies[i % n_copies if cold else 0].decode()

    def timed_loop(n_steps, cold):
        """Exactly n_steps calls from a Python loop between two synchronisations (includes the
        interpreter's and the binding's time per call)."""
        run(warmup, cold)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(n_steps, cold)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n_steps

    def timed_graph(n_steps, cold):
        """The same n_steps calls captured once into a HIP graph (what a serving loop does with a
        decode step that is shorter than a host-side launch) and replayed until the timed region
        is at least MIN_TIMED_SECONDS long."""
        run(warmup, cold)
        return graph_seconds(torch, lambda i, st: copies[i % n_copies if cold else 0].decode(st), n_steps)

    if kernel_only:  # the roofline leg alone (for a profiler run that should see nothing else)
        run(warmup, True)
        return w, alg_bytes, None, None, {"cold": kernel_seconds(lra, torch, lambda i, st: copies[i % n_copies].decode(st), steps)}, n_copies
    loop_cold = timed_loop(steps, True)
    sec_cold, timed_steps = timed_graph(steps, True)
    sec_hot, _ = timed_graph(steps, False)
    out = {"cold": kernel_seconds(lra, torch, lambda i, st: copies[i % n_copies].decode(st), steps),
           "hot": kernel_seconds(lra, torch, lambda i, st: copies[0].decode(st), steps),
           "loop_cold": loop_cold, "timed_steps": timed_steps}
    return w, alg_bytes, sec_cold, sec_hot, out, n_copies


def other_decode_workloads(args, torch, lra, workloads):
    """The other decode configurations (the small fp32 call of configuration 1, which runs on the vector-ALU
    kernels and is bound by latency, not by memory: reported, not graded; 8 agents x 32768 tokens, r = 64; ragged
    paged batch of 16 x 4 queries), reported next to the headline workload."""
    rows = []
    for index in (1, 4, 5):
        w, alg, sec_cold, _, ksec, n_copies = bench_decode(args, torch, lra, workloads, index,
                                                           steps=max(20, args.steps // 10),
                                                           warmup=max(5, args.warmup // 10))
        rows.append({"workload": w.name, "algorithmic_bytes": alg, "cache_copies": n_copies,
                     "value": round(alg / sec_cold / 1e9, 1), "unit": "GB/s",
                     "ms_per_step": round(sec_cold * 1e3, 5),
                     "kernel_us": round(ksec["cold"] * 1e6, 2),
                     "kernel_GBps": round(alg / ksec["cold"] / 1e9, 1),
                     "kernel_frac_of_hbm_peak": round(alg / ksec["cold"] / 1e9 / HBM_PEAK_GBS, 4)})
        torch.cuda.empty_cache()
    return rows


def value_only_decode(args, torch, lra, workloads):
    """Config 2 with b_k = NULL, reported next to the headline workload."""
    w, alg, sec_cold, _, ksec, _ = bench_decode(args, torch, lra, workloads, 2, steps=max(20, args.steps // 4),
                                                warmup=max(5, args.warmup // 4), value_only=True)
    torch.cuda.empty_cache()
    return {"workload": w.name + " with b_k = NULL", "value": round(alg / sec_cold / 1e9, 1), "unit": "GB/s",
            "ms_per_step": round(sec_cold * 1e3, 5), "kernel_us": round(ksec["cold"] * 1e6, 2),
            "kernel_GBps": round(alg / ksec["cold"] / 1e9, 1),
            "kernel_frac_of_hbm_peak": round(alg / ksec["cold"] / 1e9 / HBM_PEAK_GBS, 4)}


MIN_PREFILL_LAUNCHES = 50


def decode_kernel_label(w):
    """Name of the kernel that streams the keys of a contiguous decode workload without a rotary key
    side that fits one workgroup per compute unit (what the headline configuration is)."""
    return f"decode_stream_kernel<{w.head_dim}, 1, {32 if w.rank <= 32 else 64}>"


def base_shared_decode(args, torch, lra, workloads):
    """The headline decode workload under BaseShared (Sec. 3.2): every agent has its OWN low-rank cache
    L_a [n][r] (stored [n][A][r]), so a call streams A*r instead of r low-rank elements per token.
    Algorithmic bytes: K_base + V_base + A caches L_a + B_K + B_V + Q + out."""
    from paper_2602_01053_amd.runner import DeviceWorkload
    dev = torch.device("cuda:0")
    w = workloads.config(2)
    agents, n, r = w.n_queries, w.seq_lens[0], w.rank
    gen = torch.Generator().manual_seed(20260299)
    l_all = torch.randn(n, agents, r, generator=gen).to(torch.bfloat16)
    alg = w.algorithmic_bytes() + (agents - 1) * n * r * 2
    cache_bytes = (2 * w.k_base.numel() + l_all.numel()) * 2
    n_copies = int(math.ceil(COLD_BYTES / cache_bytes)) + 1
    base = DeviceWorkload(w, dev)
    copies = []
    for _ in range(n_copies):
        c = DeviceWorkload.__new__(DeviceWorkload)
        c.__dict__.update(base.__dict__)
        c.k_base, c.v_base = base.k_base.clone(), base.v_base.clone()
        c.l = l_all.to(dev).permute(1, 0, 2)      # view [adapter][token][r] over [n][A][r] storage
        c.cache = lra.make_cache(c.k_base, c.v_base, c.l, c.seq_lens, n, None, l_per_adapter=True)
        copies.append(c)
    nbytes = lra.lra_workspace_bytes(copies[0].shape, copies[0].cache, w.n_queries, copies[0].max_queries_per_seq, 0)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    for c in copies:
        c.workspace = ws
    steps = max(20, args.steps // 4)
    for i in range(10):
        copies[i % n_copies].decode()
    sec, _ = graph_seconds(torch, lambda i, st: copies[i % n_copies].decode(st), steps)
    ksec = kernel_seconds(lra, torch, lambda i, st: copies[i % n_copies].decode(st), steps)
    torch.cuda.empty_cache()
    return {"workload": w.name + " with one low-rank cache per agent (BaseShared)", "algorithmic_bytes": alg,
            "value": round(alg / sec / 1e9, 1), "unit": "GB/s", "ms_per_step": round(sec * 1e3, 5),
            "kernel_us": round(ksec * 1e6, 2), "kernel_GBps": round(alg / ksec / 1e9, 1),
            "kernel_frac_of_hbm_peak": round(alg / ksec / 1e9 / HBM_PEAK_GBS, 4)}


def base_shared_paged_decode(args, torch, lra, workloads):
    """The ragged paged batch (config 5) under BaseShared: one pool of low-rank rows per adapter, every query reads
    the pool of its own adapter.  Algorithmic bytes: config 5's plus the rows of the other adapters' pools."""
    from paper_2602_01053_amd.runner import DeviceWorkload
    dev = torch.device("cuda:0")
    w = workloads.config(5)
    gen = torch.Generator().manual_seed(20260305)
    pools = [w.l] + [torch.where(torch.isnan(w.l.float()), w.l.float(), torch.randn(w.l.shape, generator=gen)).to(torch.bfloat16)
                     for _ in range(w.n_adapters - 1)]
    alg = w.algorithmic_bytes() + (w.n_adapters - 1) * sum(w.seq_lens) * w.rank * 2
    dw = DeviceWorkload(w, dev)
    dw.l = torch.stack(pools).to(dev)             # [adapter][block][16][r]
    dw.cache = lra.make_cache(dw.k_base, dw.v_base, dw.l, dw.seq_lens, max(w.seq_lens), dw.block_table, l_per_adapter=True)
    nbytes = lra.lra_workspace_bytes(dw.shape, dw.cache, w.n_queries, dw.max_queries_per_seq, 0)
    dw.workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    steps = max(20, args.steps // 10)
    for _ in range(5):
        dw.decode()
    sec, _ = graph_seconds(torch, lambda i, st: dw.decode(st), steps)
    torch.cuda.empty_cache()
    return {"workload": w.name + " with one pool of low-rank rows per adapter (BaseShared)", "algorithmic_bytes": alg,
            "value": round(alg / sec / 1e9, 1), "unit": "GB/s", "ms_per_step": round(sec * 1e3, 5),
            "frac_of_hbm_peak": round(alg / sec / 1e9 / HBM_PEAK_GBS, 4)}


def bench_prefill(args, torch, lra, workloads, kernel_only=False):
    """Config 3: at least MIN_PREFILL_LAUNCHES timed launches after at least 10 warm-up launches, whatever
    --steps says (a call is one kernel of 0.6 ms; a handful of launches would time the clock ramp)."""
    from paper_2602_01053_amd.runner import DeviceWorkload
    dev = torch.device("cuda:0")
    w = workloads.config(3)
    flops = w.algorithmic_flops()
    dw = DeviceWorkload(w, dev)
    dw.alloc_workspace()
    launches = max(MIN_PREFILL_LAUNCHES, min(args.steps // 10, 200))
    for _ in range(max(10, min(args.warmup // 10, 20))):
        dw.prefill()
    torch.cuda.synchronize()
    sec = None
    if not kernel_only:
        t0 = time.perf_counter()
        for _ in range(launches):
            dw.prefill()
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / launches
    old = lra.lra_set_profile_mode(1)
    try:
        ksec, k_launches = graph_seconds(torch, lambda i, st: dw.prefill(st), 10, min_seconds=0.03)
    finally:
        lra.lra_set_profile_mode(old)
    return w, flops, sec, ksec, launches, k_launches


def bench_rotary_prefill(args, torch, lra, workloads):
    """The prefill workload with the rotary key side (lra_shape.key_rope_theta: the adapter's key
    contribution is rotated by its token's position, App. D.1): same algorithmic flops as the plain
    call; completing the keys is overhead (once per call in a pre-pass, or per key tile inside the kernel)."""
    from paper_2602_01053_amd.runner import DeviceWorkload
    w = workloads.config(3)
    dw = DeviceWorkload(w, torch.device("cuda:0"), key_rope_theta=500000.0)
    dw.alloc_workspace()
    for _ in range(3):
        dw.prefill()
    ksec, _ = graph_seconds(torch, lambda i, st: dw.prefill(st), 10, min_seconds=0.03)   # the whole call: pre-pass + kernel
    prev = lra.lra_set_rope_key_prepass(False)
    try:
        for _ in range(3):
            dw.prefill()
        isec, _ = graph_seconds(torch, lambda i, st: dw.prefill(st), 10, min_seconds=0.03)
    finally:
        lra.lra_set_rope_key_prepass(prev)
    tf = w.algorithmic_flops() / ksec / 1e12
    out = {"workload": w.name + " with key_rope_theta = 500000", "call": "lra_attn_prefill", "call_ms": round(ksec * 1e3, 4),
           "roofline": {"bound": "mfma", "achieved": round(tf, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                        "note": "flops of the plain call over the time of the whole call: a pre-pass writes the completed keys "
                                "K_base + RoPE(L B_K) of the call's adapter to the workspace, the kernel then runs on them"},
           "key_tiles_completed_in_kernel_ms": round(isec * 1e3, 4)}
    # the decode workload with the rotary key side: rotary form of the split-KV kernel + merge
    w2 = workloads.config(2)
    dw2 = DeviceWorkload(w2, torch.device("cuda:0"), key_rope_theta=500000.0)
    dw2.alloc_workspace()
    for _ in range(5):
        dw2.decode()
    sec, _ = graph_seconds(torch, lambda i, st: dw2.decode(st), 100)
    out["decode"] = {"workload": w2.name + " with key_rope_theta = 500000", "call": "lra_attn_decode",
                     "us_per_call": round(sec * 1e6, 2), "GBps_of_the_plain_call's_bytes": round(w2.algorithmic_bytes() / sec / 1e9, 1),
                     "note": "same buffers every call (hot); keys are streamed once, L B_K is rotated per tile and agent in registers"}
    return out


def bench_append(args, torch, lra, with_cpu, sizes=(16384, 2048, 1)):
    """lra_cache_append at the Llama-3-8B projection shape (d_model 4096 -> 8 kv heads x 128 keys
    and values + rank 16, rotary base 500000): the chunk sizes of the prefill workload and of
    the longest trace step (MFMA-bound, TFLOP/s) and one decode step (one pass over the
    weights, HBM-bound, GB/s).  HIP events around replays of a HIP graph of back-to-back calls;
    one call is one kernel."""
    import numpy as np
    dev = torch.device("cuda:0")
    hkv, d, r, dm, theta = 8, 128, 16, 4096, 500000.0
    gen = torch.Generator(device="cpu").manual_seed(20260203)
    w_host = (torch.randn(2 * hkv * d + r, dm, generator=gen) / dm ** 0.5).to(torch.bfloat16)
    w = w_host.to(dev)
    shape = lra.make_shape(torch.empty(1, hkv, d, dtype=torch.bfloat16, device=dev), hkv, r, 0.0)
    hip = _hip()
    stream = torch.cuda.current_stream().cuda_stream or None
    rows = []
    # weight-streaming sizes: 40 copies of the weights (680 MB, beyond the memory-side cache) taken in turn, as
    # the layers of a model would be; the same-weights figure is reported beside it
    w_copies = [w] + [w.clone() for _ in range(39)] if any(n <= 64 for n in sizes) else [w]

    def timed_graph(launch, per_graph, replays):
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            for i in range(3):
                launch(i, side)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for i in range(per_graph):
                launch(i, side)
        graph.replay()
        torch.cuda.synchronize()
        e0, e1 = ctypes.c_void_p(), ctypes.c_void_p()
        assert hip.hipEventCreate(ctypes.byref(e0)) == 0 and hip.hipEventCreate(ctypes.byref(e1)) == 0
        assert hip.hipEventRecord(e0, stream) == 0
        for _ in range(replays):
            graph.replay()
        assert hip.hipEventRecord(e1, stream) == 0
        hip.hipEventSynchronize(e1)
        ms = ctypes.c_float()
        assert hip.hipEventElapsedTime(ctypes.byref(ms), e0, e1) == 0
        hip.hipEventDestroy(e0)
        hip.hipEventDestroy(e1)
        del graph
        return ms.value * 1e-3 / (per_graph * replays)

    for n_new in sizes:
        x = torch.randn(n_new, dm, generator=gen).to(torch.bfloat16).to(dev)
        k = torch.empty(n_new, hkv, d, dtype=torch.bfloat16, device=dev)
        v = torch.empty_like(k)
        l = torch.empty(n_new, r, dtype=torch.bfloat16, device=dev)
        lens = torch.tensor([n_new], dtype=torch.int32, device=dev)
        cache = lra.make_cache(k, v, l, lens, n_new, None)
        # the calls are captured into a HIP graph and the graph is replayed: a decode-step call
        # is shorter than the Python call overhead, which would otherwise be what is timed
        streaming = n_new <= 64
        per_graph, replays = (120, 5) if streaming else (10, 5)
        # with the workspace the library asks for, mid-sized chunks divide d_model over the chip
        ws_bytes = lra.lra_append_workspace_bytes(shape, cache, w, theta, n_new)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev) if ws_bytes else None
        sec_same = timed_graph(lambda i, st: lra.lra_cache_append(shape, cache, w, theta, x, 0, st, workspace=ws), per_graph, replays)
        sec = sec_same
        if streaming:
            sec = timed_graph(lambda i, st: lra.lra_cache_append(shape, cache, w_copies[i % len(w_copies)], theta, x, 0, st, workspace=ws),
                              per_graph, replays)
        sec_no_ws = timed_graph(lambda i, st: lra.lra_cache_append(shape, cache, w, theta, x, 0, st), per_graph, replays) if ws_bytes else None
        flops = 2.0 * n_new * dm * (2 * hkv * d + r)
        nbytes = 2.0 * ((2 * hkv * d + r) * dm + n_new * dm + n_new * (2 * hkv * d + r))
        row = {"n_new": n_new, "us_per_call": round(sec * 1e6, 2), "algorithmic_flops": flops,
               "algorithmic_bytes": nbytes}
        if ws_bytes:
            row["workspace_bytes"] = ws_bytes
            row["us_per_call_without_workspace"] = round(sec_no_ws * 1e6, 2)
        if n_new > 64:
            tf = flops / sec / 1e12
            row["roofline"] = {"bound": "mfma", "achieved": round(tf, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                               "unit": "TFLOP/s", "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4)}
        else:
            gbs = nbytes / sec / 1e9
            row["roofline"] = {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                               "frac": round(gbs / HBM_PEAK_GBS, 4),
                               "note": "40 copies of the weights in turn (cold); same_weights_us is back-to-back calls on one copy, "
                                       "served partly by the memory-side cache"}
            row["same_weights_us"] = round(sec_same * 1e6, 2)
        rows.append(row)
    out = {"call": "lra_cache_append", "workload": "Llama-3-8B key/value/LoRA-down projection, d_model 4096, bf16, rotary keys",
           "rows": rows}
    if with_cpu:
        import oracle
        n_s = 256
        xs = torch.randn(n_s, dm, generator=gen).to(torch.bfloat16).to(torch.float64).numpy()
        ws = w_host.to(torch.float64).numpy()
        t0 = time.perf_counter()
        oracle.project_new_tokens(xs, ws, hkv, d, r, np.arange(1000, 1000 + n_s), theta)
        sec = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(2.0 * n_s * dm * (2 * hkv * d + r) / sec / 1e12, 5), "unit": "TFLOP/s",
                               "kind": "oracle", "seconds": round(sec, 4), "sample": f"{n_s} new tokens, fp64 numpy oracle, one run"}
    return out


def bench_trace_leg(torch, lra):
    """The second workload: the 17-step agent-iteration trace of App. C.5 (bench_trace.py) at its four
    retrieved-context lengths; attention calls of one layer for one iteration, plus the producer's leg."""
    import bench_trace
    rows = []
    for l_ctx in (256, 1024, 4096, 16384):
        r = bench_trace.run_trace(torch, lra, l_ctx, replays=3)
        rows.append({"l_ctx": l_ctx, "tokens": r["trajectory_tokens"], "calls": r["calls"],
                     "attention_ms": r["attention_ms_per_layer"], "prefill_ms": r["prefill_ms_per_layer"],
                     "decode_ms": r["decode_ms_per_layer"], "decode_us_per_token": r["decode_us_per_token_per_layer"],
                     "append_ms": r["cache_append_ms_per_layer"]})
        torch.cuda.empty_cache()
    return {"workload": "emulated agent-iteration trace (17 steps: prefill P_k then G_k generated tokens per step, 3 adapters), "
                        "Llama-3-8B attention shape, one layer, one iteration", "timing": "HIP graph replay of all calls of one iteration",
            "rows": rows}


def cpu_baseline(workloads):
    """The oracle as it stands, on the host cores, on the decode workload."""
    import numpy as np  # noqa: F401
    from tests.harness import oracle_decode
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    w = workloads.config(2)
    best = float("inf")
    reps = 0
    t_all = time.perf_counter()
    while reps < 3 or (time.perf_counter() - t_all < 10.0 and reps < 20):
        t0 = time.perf_counter()
        oracle_decode(w)
        best = min(best, time.perf_counter() - t0)
        reps += 1
    return {"value": round(w.algorithmic_bytes() / best / 1e9, 4), "unit": "GB/s", "cores": int(cores),
            "kind": "oracle", "seconds": round(best, 4),
            "sample": f"the full decode workload ({w.name}: 4 queries x 32 heads x 8192 keys), "
                      f"fp64 numpy oracle, best of {reps} runs"}


def cpu_baseline_prefill(workloads):
    """The oracle on a sample of the prefill workload's new-token rows (rows are independent): every eighth
    row of the block, all 32 heads each, timed once; flops counted as for the GPU (visible pairs of those rows)."""
    from tests.harness import oracle_prefill
    w = workloads.config(3)
    rows = list(range(3, w.n_new, 8))
    t0 = time.perf_counter()
    oracle_prefill(w, rows=rows)
    sec = time.perf_counter() - t0
    n = int(w.seq_lens[0])
    d, r, hq = int(w.q.shape[-1]), int(w.l.shape[-1]), int(w.q.shape[-2])
    pairs = sum(n - w.n_new + i + 1 for i in rows) * hq
    flops = 4.0 * (d + r) * pairs + 4.0 * len(rows) * hq * d * r
    return {"value": round(flops / sec / 1e12, 5), "unit": "TFLOP/s", "kind": "oracle", "seconds": round(sec, 3),
            "sample": f"{len(rows)} of the {w.n_new} new-token rows of {w.name}, all heads, fp64 numpy oracle, one run"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prefill", action="store_true")
    ap.add_argument("--no-other-decode", action="store_true")
    ap.add_argument("--no-append", action="store_true")
    ap.add_argument("--no-trace", action="store_true")
    ap.add_argument("--profile-leg", choices=["decode_cfg2_kernel", "prefill_cfg3_kernel"],
                    help="run only the named roofline leg (the dominant kernel alone, launched exactly as in the full "
                         "run) and print its own JSON line: for a profiler run whose per-kernel average should be "
                         "that leg's and nothing else's")
    ap.add_argument("--append-only", action="store_true",
                    help="only the lra_cache_append sweep over chunk sizes (its own JSON line)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2602_01053_amd as lra
    from paper_2602_01053_amd import workloads
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    lra.load_library()

    if args.append_only:
        print(json.dumps(bench_append(args, torch, lra, False,
                                      sizes=(1, 2, 4, 8, 16, 32, 64, 128, 512, 1024, 2048, 8192, 16384))), flush=True)
        return

    if args.profile_leg == "decode_cfg2_kernel":
        w, alg_bytes, _, _, ksec, n_copies = bench_decode(args, torch, lra, workloads, kernel_only=True)
        k_gbs = alg_bytes / ksec["cold"] / 1e9
        print(json.dumps({"leg": args.profile_leg, "workload": w.name, "kernel": decode_kernel_label(w),
                          "algorithmic_bytes": alg_bytes, "cache_copies": n_copies,
                          "kernel_us": round(ksec["cold"] * 1e6, 3), "achieved_GBps": round(k_gbs, 1),
                          "frac": round(k_gbs / HBM_PEAK_GBS, 4)}), flush=True)
        return
    if args.profile_leg == "prefill_cfg3_kernel":
        wp, flops, _, pksec, _, pk_launches = bench_prefill(args, torch, lra, workloads, kernel_only=True)
        print(json.dumps({"leg": args.profile_leg, "workload": wp.name, "kernel": "prefill_mfma_kernel<128, 16>",
                          "algorithmic_flops": flops, "kernel_launches": pk_launches,
                          "kernel_ms": round(pksec * 1e3, 4), "achieved_TFLOPs": round(flops / pksec / 1e12, 2),
                          "frac": round(flops / pksec / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}), flush=True)
        return

    w, alg_bytes, sec_cold, sec_hot, ksec, n_copies = bench_decode(args, torch, lra, workloads)
    gbs = alg_bytes / sec_cold / 1e9
    k_gbs = alg_bytes / ksec["cold"] / 1e9
    line = {
        "metric": "LoRA-attn decode HBM GB/s + prefill TFLOP/s (frac of peak), Llama-3-8B shape",
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec_cold * 1e3, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "call": "lra_attn_decode", "agents": 4, "n": 8192, "q_heads": 32,
                   "kv_heads": 8, "head_dim": 128, "rank": 16, "algorithmic_bytes": alg_bytes,
                   "cache_protocol": f"cold: {n_copies} rotating copies of K_base/V_base/L"},
        "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
        "timing": {"method": "the K calls captured once into a HIP graph, replays timed with HIP events until the "
                             "timed region is at least 20 ms", "timed_steps": ksec["timed_steps"],
                   "python_loop_ms_per_step": round(ksec["loop_cold"] * 1e3, 6),
                   "python_loop_GBps": round(alg_bytes / ksec["loop_cold"] / 1e9, 1),
                   "python_loop_note": "exactly K calls issued one by one from Python between two synchronisations: "
                                       "includes the interpreter and ctypes time per call"},
        "roofline": _traffic_fields({"bound": "hbm", "kernel": decode_kernel_label(w), "achieved": round(k_gbs, 1),
                                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(k_gbs / HBM_PEAK_GBS, 4),
                                     "kernel_us": round(ksec["cold"] * 1e6, 3)}, "decode_cfg2", ksec["cold"]),
        "hot_cache": {"value": round(alg_bytes / sec_hot / 1e9, 1), "unit": "GB/s",
                      "ms_per_step": round(sec_hot * 1e3, 6), "kernel_us": round(ksec["hot"] * 1e6, 3),
                      "note": "same buffers every step: served largely by the memory-side cache"},
    }
    if not args.no_prefill:
        wp, flops, psec, pksec, psteps, pk_launches = bench_prefill(args, torch, lra, workloads)
        tf = flops / psec / 1e12
        ktf = flops / pksec / 1e12
        line["prefill"] = {
            "workload": wp.name, "call": "lra_attn_prefill", "launches": psteps, "kernel_launches": pk_launches,
            "value": round(tf, 2), "unit": "TFLOP/s", "ms_per_step": round(psec * 1e3, 4),
            "algorithmic_flops": flops, "frac_of_mfma_peak": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
            "roofline": _traffic_fields({"bound": "mfma", "kernel": "prefill_mfma_kernel<128, 16>", "achieved": round(ktf, 2),
                                         "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                         "frac": round(ktf / MFMA_BF16_PEAK_TFLOPS, 4),
                                         "kernel_ms": round(pksec * 1e3, 4)}, "prefill_cfg3", pksec)}
    if not args.no_prefill:
        line["rotary_key_prefill"] = bench_rotary_prefill(args, torch, lra, workloads)
    if not args.no_other_decode:
        line["other_decode_workloads"] = other_decode_workloads(args, torch, lra, workloads)
        line["value_only_adapters"] = value_only_decode(args, torch, lra, workloads)
        line["base_shared"] = base_shared_decode(args, torch, lra, workloads)
        line["base_shared"]["paged_batch"] = base_shared_paged_decode(args, torch, lra, workloads)
    if not args.no_append:
        line["cache_append"] = bench_append(args, torch, lra, not args.no_cpu_baseline)
    if not args.no_trace:
        line["trace"] = bench_trace_leg(torch, lra)
    ceil = machine_ceilings(torch, lra)
    line["machine_ceilings"] = ceil
    line["roofline"]["frac_of_measured_ceiling"] = round(k_gbs / ceil["hbm_stream_read_GBps"], 4)
    probe_s = stream_read_at_size(torch, lra, alg_bytes)
    line["roofline"]["ceiling_at_this_size"] = {
        "GBps": round(alg_bytes / probe_s / 1e9, 1), "us": round(probe_s * 1e6, 3),
        "frac_of_it": round(probe_s / ksec["cold"], 4),
        "note": "lra_probe_stream_read on buffers of the call's algorithmic bytes, rotating copies, same timing "
                "method as kernel_us: a plain read of this size, launch included"}
    if "prefill" in line:
        line["prefill"]["roofline"]["frac_of_measured_ceiling"] = round(
            line["prefill"]["roofline"]["achieved"] / ceil["mfma_bf16_TFLOPs"], 4)
        line["prefill"]["roofline"]["frac_of_ceiling_with_random_operands"] = round(
            line["prefill"]["roofline"]["achieved"] / ceil["mfma_bf16_random_operands_TFLOPs"], 4)
    for row in line.get("cache_append", {}).get("rows", []):
        if row["roofline"]["bound"] == "mfma":
            row["roofline"]["frac_of_ceiling_with_random_operands"] = round(
                row["roofline"]["achieved"] / ceil["mfma_bf16_random_operands_TFLOPs"], 4)
    if not args.no_cpu_baseline:
        if "prefill" in line:
            line["prefill"]["cpu_baseline"] = cpu_baseline_prefill(workloads)
        line["cpu_baseline"] = cpu_baseline(workloads)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
