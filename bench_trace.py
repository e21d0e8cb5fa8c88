#!/usr/bin/env python3
"""Second workload: the agent-iteration trace of LRAgent (App. C.5 "Emulated Trace for
Efficiency Analysis", the table of prefill and generation lengths per agent step) driven
through lra_attn_prefill / lra_attn_decode at the Llama-3-8B attention shape.

One iteration is 17 agent steps (five plan-plan-action cycles, two reflect steps).  Step k
appends P_k context tokens (one causal prefill call by that step's agent) and then
generates G_k tokens (G_k single-query decode calls, the context growing by one each).
The producer of the caches (lra_cache_append: one call per prefill chunk and per generated
token, Llama-3-8B projection shape) is timed as a separate leg over the same schedule, with
40 copies of the projection weights taken in turn so that every call reads them from HBM, as
a layer of a model does (its other layers' weights pass through the caches in between).
The retrieved-context length L_ctx sets four of the P_k.  Only attention is timed - this
library holds no projections or MLPs - so the figures are the attention share of one layer
for one iteration, not the paper's end-to-end throughput; shapes only, random data.

All calls of an iteration are captured once into a HIP graph on a side stream and replayed,
so the time is GPU time without the Python call overhead between the ~300 launches.

Prints ONE JSON line.  `python bench_trace.py [--replays N] [--lctx 256,1024,...] [--key-rope-theta 500000]`
"""
import argparse
import json
import sys

# (agent, prefill, generation); None stands for L_ctx
TRACE = [("plan", 512, 32), ("plan", 8, 8), ("action", 8, 8)]
for _ in range(4):
    TRACE += [("plan", None, 32), ("plan", 8, 8), ("action", 8, 8)]
TRACE += [("reflect", 32, 32), ("reflect", 8, 8)]
ADAPTER = {"plan": 0, "action": 1, "reflect": 2}
HQ, HKV, D, R, LAYERS = 32, 8, 128, 16, 32
D_MODEL, ROPE_THETA = 4096, 500000.0


def run_trace(torch, lra, l_ctx, replays, key_rope_theta=0.0):
    dev = torch.device("cuda:0")
    steps = [(a, l_ctx if p is None else p, g) for a, p, g in TRACE]
    total = sum(p + g for _, p, g in steps)
    gen = torch.Generator(device="cpu").manual_seed(20260201 + l_ctx)
    bf = torch.bfloat16
    k_base = torch.randn(total, HKV, D, generator=gen).to(bf).to(dev)
    v_base = torch.randn(total, HKV, D, generator=gen).to(bf).to(dev)
    l = torch.randn(total, R, generator=gen).to(bf).to(dev)
    b_k = (0.02 * torch.randn(3, R, HKV * D, generator=gen)).to(bf).to(dev)
    b_v = (0.02 * torch.randn(3, R, HKV * D, generator=gen)).to(bf).to(dev)
    max_p = max(p for _, p, _ in steps)
    q = torch.randn(max_p, HQ, D, generator=gen).to(bf).to(dev)
    out = torch.empty_like(q)
    # the producer of the caches: hidden states of the new tokens and [W_K; W_V; A]
    x = torch.randn(max_p, D_MODEL, generator=gen).to(bf).to(dev)
    w_cat = (torch.randn(2 * HKV * D + R, D_MODEL, generator=gen) / D_MODEL ** 0.5).to(bf).to(dev)
    # 40 copies taken in turn (680 MB, beyond the caches): between two appends of one layer a model reads the
    # weights of all its other layers, so a layer's projection weights come from HBM every time
    w_copies = [w_cat] + [w_cat.clone() for _ in range(39)]
    # one device int per call holds the sequence length of that call
    calls = []  # (kind, n_after, n_new, adapter)
    n = 0
    for agent, p, g in steps:
        n += p
        calls.append(("prefill", n, p, ADAPTER[agent]))
        for _ in range(g):
            n += 1
            calls.append(("decode", n, 1, ADAPTER[agent]))
    lens = torch.tensor([c[1] for c in calls], dtype=torch.int32, device=dev)
    adapters_dev = torch.tensor([0, 1, 2], dtype=torch.int32, device=dev)
    qstart = torch.tensor([0, 1], dtype=torch.int32, device=dev)
    shape = lra.make_shape(q, HKV, R, 0.0, key_rope_theta)
    ws_bytes = 256
    aws_bytes = 256   # lra_cache_append's own workspace (mid-sized chunks divide d_model over the chip)
    prepared = []
    for i, (kind, n_after, n_new, a) in enumerate(calls):
        cache = lra.make_cache(k_base, v_base, l, lens[i:i + 1], n_after, None)
        if kind == "prefill":
            ws_bytes = max(ws_bytes, lra.lra_workspace_bytes(shape, cache, 1, 1, n_new))
        else:
            ws_bytes = max(ws_bytes, lra.lra_workspace_bytes(shape, cache, 1, 1, 0))
        aws_bytes = max(aws_bytes, lra.lra_append_workspace_bytes(shape, cache, w_cat, ROPE_THETA, n_new))
        prepared.append((kind, cache, n_new, a))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    aws = torch.empty(aws_bytes, dtype=torch.uint8, device=dev)

    def iteration(stream, only=None):
        for i, (kind, cache, n_new, a) in enumerate(prepared):
            if only == "append":
                lra.lra_cache_append(shape, cache, w_copies[i % len(w_copies)], ROPE_THETA, x[:n_new], 0, stream, workspace=aws)
                continue
            if only is not None and kind != only:
                continue
            if kind == "prefill":
                lra.lra_attn_prefill(shape, cache, b_k, b_v, 3, q[:n_new], 0, a, out[:n_new], ws, stream)
            else:
                lra.lra_attn_decode(shape, cache, b_k, b_v, 3, q[:1], adapters_dev[a:a + 1], qstart, 1, out[:1], ws, stream)

    side = torch.cuda.Stream()
    res = {}
    for label, only in (("all", None), ("prefill", "prefill"), ("decode", "decode"), ("append", "append")):
        with torch.cuda.stream(side):
            iteration(side, only)  # warm-up outside the graph
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            iteration(side, only)
        graph.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(replays):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
        res[label] = e0.elapsed_time(e1) / replays  # ms per iteration, one layer
    n_prefill = sum(p for _, p, _ in steps)
    n_gen = sum(g for _, _, g in steps)
    return {"l_ctx": l_ctx, "trajectory_tokens": total, "prefill_tokens": n_prefill, "generated_tokens": n_gen,
            "calls": len(calls), "attention_ms_per_layer": round(res["all"], 4),
            "prefill_ms_per_layer": round(res["prefill"], 4), "decode_ms_per_layer": round(res["decode"], 4),
            "attention_ms_32_layers": round(res["all"] * LAYERS, 3),
            "cache_append_ms_per_layer": round(res["append"], 4),
            "decode_us_per_token_per_layer": round(res["decode"] * 1e3 / n_gen, 2)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--replays", type=int, default=5)
    ap.add_argument("--lctx", type=str, default="256,1024,4096,16384")
    ap.add_argument("--key-rope-theta", type=float, default=0.0,
                    help="> 0: the rotary key side (LoRA on the key projection, App. D.1) with this base")
    args = ap.parse_args()
    import torch
    import paper_2602_01053_amd as lra
    if not torch.cuda.is_available():
        print("bench_trace.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    lra.load_library()
    rows = [run_trace(torch, lra, int(x), args.replays, args.key_rope_theta) for x in args.lctx.split(",")]
    print(json.dumps({"workload": "LRAgent emulated agent-iteration trace (17 steps), attention only, "
                                  "Llama-3-8B attention shape (32 q / 8 kv heads, d=128, r=16), bf16, one sequence, 3 adapters",
                      "key_rope_theta": args.key_rope_theta, "data": "synthetic", "timing": "HIP graph replay of all calls of one iteration",
                      "rows": rows}), flush=True)


if __name__ == "__main__":
    main()
