#!/usr/bin/env python3
"""Benchmark of the whole-model decode kernel on one MI355X.

A "step" is one decode step (one token per sequence) of the whole hot path: embedding gather,
all layers (RMSNorm, QKV projection, RoPE, cache append, split-KV attention + merge, output
projection, SwiGLU FFN, residuals), final norm and LM head -- one persistent kernel launch.

Default workload: Llama-3-8B-shaped decoder, bf16 random weights, batch 1, KV context 1024
(synthetic: seeded generators stand in for the Llama-3.1 checkpoint and prompts the paper used).
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per fused launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, each scaled by
# a plain copy of known size); the summary under profiles/ gives the commands and the raw figures.
def measured_traffic(workload):
    """traffic_bytes_per_launch of the workload's committed rocprofv3 summary, if it has one."""
    path = os.path.join(ROOT, "profiles", f"fused_decode_kernel_{workload}.md")
    if not os.path.isfile(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch="):
            return float(line.split("=", 1)[1])
    return None

WORKLOADS = {
    # name: (shape, wdtype, batch, context)
    "tiny-bf16-b1-ctx128": ("tiny", 0, 1, 128),
    "llama3-8b-bf16-b1-ctx1024": ("llama3-8b", 0, 1, 1024),
    "llama3-8b-bf16-b8-ctx1024": ("llama3-8b", 0, 8, 1024),     # one wide pass
    "llama3-8b-bf16-b16-ctx1024": ("llama3-8b", 0, 16, 1024),   # one wide pass
    "llama3-8b-int8-b1-ctx4096": ("llama3-8b", 1, 1, 4096),
    "llama3-8b-int8-b16-ctx4096": ("llama3-8b", 1, 16, 4096),   # one wide pass (int8 codes converted to bf16 in registers)
    "llama3-8b-int4-b1-ctx2048": ("llama3-8b", 2, 1, 2048),
    "llama3-8b-int4-b4-ctx2048": ("llama3-8b", 2, 4, 2048),
    "llama3-8b-int4-b16-ctx2048": ("llama3-8b", 2, 16, 2048),   # one wide pass (int4 codes as bf16 128 + n on the matrix cores)
    # the full 80-layer model: 139 GB of packed weights, generated and packed layer by layer on the GPU
    "llama3-70b-bf16-b1-ctx2048": ("llama3-70b", 0, 1, 2048),
    "llama3-70b-bf16-b16-ctx2048": ("llama3-70b", 0, 16, 2048),
    "llama3-70b-int4-b1-ctx2048": ("llama3-70b", 2, 1, 2048),   # the paper's largest configuration (int4 group-128, 35 GB)
}


def cpu_baseline(shape, wdtype, ctx, seed, n_layers_sample=16, steps=16, gen_device="cpu"):
    """Times the CPU oracle (as it stands) on a bounded sample: `steps` decode steps of an
    n_layers_sample-layer model of the same shape plus the LM head, scaled to the full depth."""
    import numpy as np
    from oracle import oracle
    from paper_2505_22758_amd import synth
    n_layers_sample = min(n_layers_sample, shape.n_layers)   # 8B shape: about 10 s of CPU work on 16 cores
    sub = shape.replace(n_layers=n_layers_sample)
    def to_cpu(obj):
        return {k: to_cpu(v) for k, v in obj.items()} if isinstance(obj, dict) else obj.cpu()

    # the seeded generators give identical bits on either device; generating on the GPU is faster
    layers = [to_cpu(synth.make_layer(sub, seed, l, wdtype, gen_device)) for l in range(n_layers_sample)]
    head = to_cpu(synth.make_head(sub, seed, wdtype, gen_device))
    M = oracle.OracleModel(sub, layers, head)
    kv = M.new_kv(1, ctx + steps)
    for l in range(n_layers_sample):
        k, v = synth.make_kv_prefill(sub, seed, l, 0, ctx, gen_device)
        kv[l, 0, 0, :ctx], kv[l, 0, 1, :ctx] = oracle._np(k.cpu()), oracle._np(v.cpu())
    toks = synth.make_tokens(sub, seed, steps, 1)
    x = M.embed(int(toks[0, 0]))
    t_layers = t_head = 0.0
    for s in range(steps):
        x = M.embed(int(toks[s, 0]))
        t0 = time.perf_counter()
        for l in range(n_layers_sample):
            M.layer_step(l, x, kv[l, 0, 0], kv[l, 0, 1], ctx + s)
        t1 = time.perf_counter()
        M.logits(x)
        t2 = time.perf_counter()
        t_layers += t1 - t0
        t_head += t2 - t1
    per_step = (t_layers / n_layers_sample * shape.n_layers + t_head) / steps
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": per_step * 1e6, "unit": "us/token", "cores": cores, "kind": "oracle",
            "sample": f"{steps} step(s) of {n_layers_sample} of {shape.n_layers} layers + LM head at full width, "
                      f"ctx {ctx}; per-layer time x {shape.n_layers} + head time"}


def stack_ablation(args):
    """The paper's component studies on this machine (Section 3: stacked square linear layers;
    Section 5.3: stacked attention and GLU blocks): Baseline (one launch per operation) / Fused (one
    persistent kernel, tiles requested after the input has arrived) / + Overlap (tiles requested before
    the input is waited for).  Prints one JSON line per cell."""
    import numpy as np
    import torch
    from paper_2505_22758_amd import binding, synth
    dev = "cuda:0"
    torch.cuda.set_device(0)
    reps = args.steps

    def timed(fn):
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3   # us

    def graphed(fn):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return timed(g.replay)

    layers_list = [int(v) for v in args.layers.split(",")]
    if args.stack == "linear":
        for d in [int(v) for v in args.dim.split(",")]:
            for L in layers_list:
                w = synth.normal_bf16(7, f"stack{d}", (L, d, d), 0.02, dev)
                x = synth.normal_bf16(7, "stack.x", (d,), 1.0, dev).float()
                y = torch.empty_like(x)
                scratch = torch.zeros(2 * ((4 * d + 255) // 256 * 256) + 256, dtype=torch.uint8, device=dev)
                cell = {"stack": "linear", "dim": d, "layers": L, "weight_bytes": 2 * L * d * d}
                for mode, name in ((0, "baseline"), (1, "fused"), (2, "fused+overlap")):
                    us = timed(lambda: binding.ff_debug_stack_linear(w, x, y, mode, scratch))
                    cell[name + "_us"] = us
                    cell[name + "_gbs"] = cell["weight_bytes"] / us / 1e3
                cell["baseline_graph_us"] = graphed(lambda: binding.ff_debug_stack_linear(w, x, y, 0, scratch))
                assert int(scratch[-256:].view(torch.int32)[0]) == 0, "a stacked-linear launch recorded a time-out"
                print(json.dumps(cell), flush=True)
                del w
                torch.cuda.empty_cache()
        return
    base = synth.SHAPES["llama3-8b"]
    if args.stack == "attn":     # attention sublayer with a vestigial FFN (d_ffn 128: 0.4 % of the layer's bytes)
        shape, ctx = base.replace(name="stack-attn", d_ffn=128, vocab=256), 1024
    else:                        # GLU sublayer with a vestigial attention (4 query / 1 kv head of 128, one cached row: 3 % of the bytes)
        shape, ctx = base.replace(name="stack-glu", n_q_heads=4, n_kv_heads=1, vocab=256), 1
    for L in layers_list:
        S = shape.replace(n_layers=L)
        dec = binding.Decoder.synthetic(S, 11, synth.WDTYPE_BF16, 1, device=dev)
        dec.alloc_kv(1, ctx + 4)
        binding.ff_kv_fill_synthetic(dec.kv, 11, ctx)
        tok = torch.tensor([5], dtype=torch.int32, device=dev)
        pos = torch.tensor([ctx], dtype=torch.int32, device=dev)
        lg = torch.zeros(1, S.vocab, device=dev)
        wbytes = synth.weight_bytes_per_step(S, synth.WDTYPE_BF16) + synth.kv_bytes_per_step(S, 1, ctx)
        cell = {"stack": args.stack, "layers": L, "bytes_per_step": wbytes}
        cell["baseline_us"] = timed(lambda: dec.step(tok, pos, lg, perop=True))
        cell["baseline_graph_us"] = graphed(lambda: dec.step(tok, pos, lg, perop=True))
        binding.ff_debug_set_overlap(dec.model, False)
        cell["fused_us"] = timed(lambda: dec.step(tok, pos, lg))
        binding.ff_debug_set_overlap(dec.model, True)
        cell["fused+overlap_us"] = timed(lambda: dec.step(tok, pos, lg))
        binding.ff_status(dec.model)
        for k in ("baseline", "fused", "fused+overlap"):
            cell[k + "_gbs"] = wbytes / cell[k + "_us"] / 1e3
        print(json.dumps(cell), flush=True)
        dec.close()
        del dec
        torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="llama3-8b-bf16-b1-ctx1024", choices=sorted(WORKLOADS))
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch (sweeps)")
    ap.add_argument("--ctx", type=int, default=0, help="override the workload's KV context (sweeps)")
    ap.add_argument("--ctx-list", default="", help="one KV context per sequence, comma separated (ragged batch; overrides --batch and --ctx)")
    ap.add_argument("--uniform-attention-shares", action="store_true",
                    help="attention work list with the same number of workgroups for every sequence (default: by length)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-perop", action="store_true")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the streaming-read ceiling measurement")
    ap.add_argument("--stack", choices=["linear", "attn", "glu"], help="component ablation instead of the decode benchmark")
    ap.add_argument("--dim", default="2048,4096,8192", help="--stack linear: widths")
    ap.add_argument("--layers", default="1,4,32", help="--stack: depths")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (a known-traffic kernel to scale rocprofv3 --pmc counters by)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the paper's kernel is single-GPU); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)

    if args.stack:
        return stack_ablation(args)

    import numpy as np
    import torch
    from paper_2505_22758_amd import binding, synth

    shape_name, wdtype, batch, ctx = WORKLOADS[args.workload]
    batch, ctx = args.batch or batch, args.ctx or ctx
    ctxs = [int(v) for v in args.ctx_list.split(",")] if args.ctx_list else [ctx] * batch   # rows cached per sequence before the first step
    batch, ctx = len(ctxs), max(ctxs)
    shape = synth.SHAPES[shape_name]
    seed = 0x250522758
    dev = "cuda:0"
    torch.cuda.set_device(0)
    total_steps = args.warmup + args.steps
    max_ctx = ctx + total_steps + 1

    # weights and cache prefill: the library's device-side generator (same bits as synth.py, tested)
    dec = binding.Decoder.synthetic(shape, seed, wdtype, max_batch=batch, device=dev)
    if args.uniform_attention_shares:
        binding.ff_debug_set_attention_balance(dec.model, False)
    torch.cuda.synchronize()

    def new_cache():
        buf = torch.zeros(binding.ff_kv_bytes(dec.model, batch, max_ctx), dtype=torch.uint8, device=dev)
        kv = binding.ff_kv_alloc(dec.model, batch, max_ctx, buf)
        binding.ff_kv_fill_synthetic(kv, seed, ctx)
        torch.cuda.synchronize()
        return kv, buf

    toks = synth.make_tokens(shape, seed, total_steps, batch).to(dev)
    pos = (torch.arange(total_steps, dtype=torch.int32, device=dev)[:, None] + torch.tensor(ctxs, dtype=torch.int32, device=dev)[None, :]).contiguous()
    logits = torch.zeros(batch, shape.vocab, dtype=torch.float32, device=dev)

    def run(fn, kv, n0, n):
        """Run steps [n0, n0+n); returns (wall ms for all, per-step event ms list)."""
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        evs[0].record()
        for i in range(n):
            fn(dec.model, toks[n0 + i], pos[n0 + i], kv, logits, batch)
            evs[i + 1].record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3
        return wall, [evs[i].elapsed_time(evs[i + 1]) for i in range(n)]

    if args.calibrate_copy:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev)   # 1 GiB read + 1 GiB written
        b = torch.empty_like(a)
        a.fill_(1.0)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b
        torch.cuda.empty_cache()

    # streaming-read ceiling of this machine (what a kernel that only streams 4 GiB achieves)
    ceiling_gbs = None
    if not args.no_ceiling:
        probe = torch.empty(1 << 30, dtype=torch.float32, device=dev)   # 4 GiB
        probe.fill_(1.0)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(2):
            binding.ff_debug_stream_read(probe)
        e0.record()
        for _ in range(5):
            binding.ff_debug_stream_read(probe)
        e1.record()
        torch.cuda.synchronize()
        ceiling_gbs = 5 * probe.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del probe
        torch.cuda.empty_cache()

    kv, kv_buf = new_cache()
    run(binding.ff_decode_step, kv, 0, args.warmup)
    wall_ms, per_step_ms = run(binding.ff_decode_step, kv, args.warmup, args.steps)
    binding.ff_status(dec.model)
    ms_per_step = wall_ms / args.steps
    kern_ms = float(np.mean(per_step_ms))   # one kernel per step: event spacing = launch duration + gap

    wbytes = synth.weight_bytes_per_step(shape, wdtype)
    kvb = [sum(synth.kv_bytes_per_step(shape, 1, c + args.warmup + i) for c in ctxs) for i in range(args.steps)]
    alg_bytes = wbytes + float(np.mean(kvb))
    achieved = alg_bytes / (kern_ms * 1e-3) / 1e9

    out = {
        "metric": "per-token decode latency", "value": ms_per_step * 1e3, "unit": "us",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": {0: "bf16", 1: "int8", 2: "int4"}[wdtype] + " weights, f32 accumulate; "
                 + ("activations exchanged between phases and multiplied as bf16 head + bf16 remainder (17 bits), residual stream f32" if batch > 4
                    else "activations exchanged between phases as f32 rounded to 22 mantissa bits"
                         + ("" if batch == 1 else ", staged projection inputs as bf16 head + bf16 remainder (17 bits)")),
        "data": "synthetic",
        "config": {"workload": args.workload if not (args.batch or args.ctx or args.ctx_list) else f"{args.workload} with batch {batch}, ctx {ctx}",
                   "batch": batch, "kv_context": ctx if not args.ctx_list else ctxs,
                   "attention_shares": "equal" if args.uniform_attention_shares else "by length",
                   "weight_bytes_per_step": wbytes, "kv_bytes_per_step_mean": float(np.mean(kvb))},
        "tokens_per_s": batch / (ms_per_step * 1e-3),
        "latency_us_p10_p50_p90": [float(np.percentile(per_step_ms, q)) * 1e3 for q in (10, 50, 90)],
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None if (args.batch or args.ctx or args.ctx_list) else measured_traffic(args.workload),
                     "kernel": "fused_decode_kernel", "kernel_ms": kern_ms, "algorithmic_bytes": alg_bytes,
                     "ceiling_gbs": ceiling_gbs, "frac_of_ceiling": None if ceiling_gbs is None else achieved / ceiling_gbs},
    }

    if not args.no_perop:
        kv2, kv2_buf = new_cache()
        n_po = min(args.steps, 16)
        run(binding.ff_decode_step_perop, kv2, 0, min(args.warmup, 4))
        w_po, _ = run(binding.ff_decode_step_perop, kv2, args.warmup, n_po)
        out["perop_baseline"] = {"us_per_token": w_po / n_po * 1e3, "launches_per_step": 10 * shape.n_layers + 3,
                                 "mode": "plain stream"}
        # the same launches replayed from a HIP graph (the paper's baselines ran with graphs enabled)
        try:
            g = torch.cuda.CUDAGraph()
            gi = min(args.warmup + n_po, total_steps - 1)
            st_tok, st_pos = toks[gi].clone(), pos[gi].clone()
            with torch.cuda.graph(g):
                binding.ff_decode_step_perop(dec.model, st_tok, st_pos, kv2, logits, batch)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(n_po):
                g.replay()
            torch.cuda.synchronize()
            out["perop_baseline"]["graph_us_per_token"] = (time.perf_counter() - t0) / n_po * 1e6
        except Exception as e:  # graphs are a courtesy figure; the plain-stream number stands
            out["perop_baseline"]["graph_error"] = str(e)[:200]
        binding.ff_status(dec.model)

    if not args.no_cpu_baseline:
        dec.close()
        del dec
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(shape, wdtype, ctx, seed, gen_device=dev)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
