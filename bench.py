"""Benchmark of the MeteoRA linear-layer forward on one MI355X.

A "step" is one call of the whole layer over one batch of the workload (all stages of the hot
path: gate, top-k, bucketing, shrink, base GEMM, expand).  The weights are static during inference,
so their kernel-side layouts are packed once before the timed region (meteora_pack_weights) and
every step calls meteora_linear_forward_packed; the same loop with per-call packing
(meteora_linear_forward) is timed as well and reported beside it.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--layer 0] [--tokens T] [--no-cpu-baseline] [--graph]

The defaults (1000 timed steps after 100 warm-up steps, about 0.15 s) reach the steady state of the
clocks; runs of a few dozen steps measure 4-5% slower.  --graph also replays the step from a captured
HIP graph (works, tested; eager enqueue is faster because the host stays ahead of the GPU).

--tokens T runs the configuration's layer shapes with T tokens instead of its own batch (for the batch sizes
between decode and prefill; the headline workload is the configuration's own T).

--layer -1 runs every layer of the configuration one after the other per step (config 5: the seven
projections of a Llama3-8B block, each a MeteoRA layer with its own gate and adapters, fed the same
number of tokens); tokens/s is then T / (time of the whole set), and the roofline figures are those of
the set's GEMM launches together.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E

# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of
# this same command (each counter scaled by what it reads for a plain 1 GiB copy kernel: 2.0 and 1.0);
# the summary is profiles/linear_forward_config2_hbm_traffic.md.  Only the profiled workload has a value.
MEASURED_GEMM_TRAFFIC_BYTES = {(2, 0): 106856.5 * 2.0 * 1024 + 37376.0 * 1024}


def algorithmic(shape):
    """Algorithmic flops and bytes of each stage of one layer call (e = bytes per element)."""
    s = shape
    e = 2 if s.dtype == "bf16" else 4
    T, di, do, N, r, k = s.T, s.d_in, s.d_out, s.N, s.r, s.k
    return {
        "gate": {"flops": 2.0 * T * di * N, "bytes": T * di * e + di * N * 4 + T * k * 8},
        "shrink": {"flops": 2.0 * T * k * di * r, "bytes": T * di * e + N * di * r * e + T * k * r * 4},
        "expand": {"flops": 2.0 * T * k * r * do, "bytes": T * k * r * 4 + N * r * do * e + T * do * e},
        "gemm": {"flops": 2.0 * T * di * do, "bytes": T * di * e + di * do * e + T * do * e},
    }


def cpu_baseline(shape, ops, budget_s=15.0):
    """Time the CPU oracle (as it stands) on a bounded sample of rows of the same workload."""
    import numpy as np
    import oracle
    probe = np.arange(0, shape.T, max(1, shape.T // 16), dtype=np.int32)[:16]
    t0 = time.perf_counter()
    oracle.linear_forward(ops["x"], ops["W"], ops["W_gate"], ops["bias"], ops["A"], ops["B"], shape.k, shape.scale,
                          rows=probe)
    per_row = (time.perf_counter() - t0) / probe.size
    n = int(max(16, min(shape.T, budget_s / max(per_row, 1e-9))))
    rows = np.linspace(0, shape.T - 1, n).astype(np.int32)
    t0 = time.perf_counter()
    oracle.linear_forward(ops["x"], ops["W"], ops["W_gate"], ops["bias"], ops["A"], ops["B"], shape.k, shape.scale,
                          rows=rows)
    dt = time.perf_counter() - t0
    return {"value": n / dt, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{n} of {shape.T} token rows (evenly strided) of the same layer, {dt:.1f} s wall"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--layer", type=int, default=0)
    ap.add_argument("--tokens", type=int, default=0,
                    help="run the configuration's layer shapes with this many tokens instead of its own T")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step replayed from a captured HIP graph (reported as hip_graph)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
                 "(the layer shards by tokens with no exchange step between the GPUs)")

    import numpy as np
    import torch
    import paper_2405_13053_amd as m
    from gen import inputs as gen

    torch.cuda.set_device(0)
    seed, layers = gen.config_layers(args.config)
    if args.tokens > 0:
        import dataclasses
        layers = [dataclasses.replace(sh, T=args.tokens) for sh in layers]
    which = list(range(len(layers))) if args.layer < 0 else [args.layer]
    dt_of = lambda sh: torch.bfloat16 if sh.dtype == "bf16" else torch.float32
    calls = []   # one entry per layer: everything a call needs, resident on the GPU
    for li in which:
        sh = layers[li]
        ops_l = gen.make_layer(sh, seed, li)
        dt = dt_of(sh)
        dev = {n: torch.from_numpy(ops_l[n]).cuda().to(dt) for n in ("x", "W", "A", "B")}
        Wg = torch.from_numpy(ops_l["W_gate"]).cuda()
        bias = None if ops_l["bias"] is None else torch.from_numpy(ops_l["bias"]).cuda()
        out = torch.empty((sh.T, sh.d_out), dtype=dt, device="cuda")
        ws = torch.empty(m.workspace_bytes(sh.T, sh.d_in, sh.d_out, sh.N, sh.r, sh.k, dt), dtype=torch.uint8,
                         device="cuda")
        packed = m.pack_weights(Wg, dev["A"], dev["B"])   # once per set of adapters, outside the timed region
        calls.append((sh, dev, Wg, bias, out, ws, packed))
        if li == which[0]:
            ops = ops_l   # the CPU baseline samples the first layer
    shape = calls[0][0]

    def step():
        for sh, dev, Wg, bias, out, ws, packed in calls:
            m.linear_forward(dev["x"], dev["W"], Wg, bias, dev["A"], dev["B"], sh.k, sh.scale, out=out, ws=ws,
                             packed=packed)

    def step_repack():
        for sh, dev, Wg, bias, out, ws, packed in calls:
            m.linear_forward(dev["x"], dev["W"], Wg, bias, dev["A"], dev["B"], sh.k, sh.scale, out=out, ws=ws)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    elapsed_repack = timed(step_repack)
    elapsed = timed(step)
    graph_ms = None
    if args.graph:
        # the library allocates nothing and records no memset, so a step can be captured once and replayed
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step()
        graph_ms = timed(graph.replay) * 1e3 / args.steps
    ms_per_step = elapsed * 1e3 / args.steps
    tokens_per_s = shape.T * args.steps / elapsed

    # per-stage durations from hipEvents recorded by the library on the launch stream (per step: summed over the
    # layers of the set)
    m.stage_timing_enable(True)
    n_prof = max(1, min(args.steps, 200 // len(calls)))
    for _ in range(n_prof):
        step()
    torch.cuda.synchronize()
    stages, _ = m.stage_timing_read()
    m.stage_timing_enable(False)
    stage_us = {n: ms * 1e3 / n_prof for n, (ms, c) in stages.items() if c > 0}

    alg = {}
    for sh, *_ in calls:
        for key, d in algorithmic(sh).items():
            acc = alg.setdefault(key, {"flops": 0.0, "bytes": 0.0})
            acc["flops"] += d["flops"]
            acc["bytes"] += d["bytes"]
    gemm_us = stage_us["gemm"]
    gemm_flops = alg["gemm"]["flops"] + (alg["expand"]["flops"] if "expand" not in stage_us else 0.0)
    achieved = gemm_flops / (gemm_us * 1e-6) / 1e12
    roofline = {"kernel": "base GEMM (bf16 MFMA)" if shape.dtype == "bf16" else "base GEMM (fp32)",
                "bound": "mfma", "achieved": achieved, "peak": PEAK_MFMA_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_MFMA_BF16_TFLOPS,
                "traffic": None if args.tokens > 0 else MEASURED_GEMM_TRAFFIC_BYTES.get((args.config, args.layer)),
                "algorithmic_bytes": alg["gemm"]["bytes"], "us": gemm_us}
    per_stage = {}
    # mid-sized batches: one launch computes the gate logits and the shrink (no bucket / shrink stage is timed);
    # its algorithmic work is the gate's plus the selected adapters' shrink, with x read once
    dense_route = "shrink" not in stage_us and "gate_logits" in stage_us
    if dense_route:
        alg["gate+shrink"] = {"flops": alg["gate"]["flops"] + alg["shrink"]["flops"],
                              "bytes": alg["gate"]["bytes"] + alg["shrink"]["bytes"] -
                                       sum(sh.T * sh.d_in * (2 if sh.dtype == "bf16" else 4) for sh, *_ in calls)}
    for n, us in stage_us.items():
        key = {"gate_logits": "gate+shrink" if dense_route else "gate", "gate_topk": None, "bucket": None}.get(n, n)
        d = {"us": round(us, 2)}
        if n == "gate_logits" and dense_route:
            d["covers"] = "gate logits and LoRA shrink in one launch; gate_topk = top-k, softmax and selection"
        if key and key in alg:
            d["GB/s"] = round(alg[key]["bytes"] / (us * 1e-6) / 1e9, 1)
            d["TFLOP/s"] = round(alg[key]["flops"] / (us * 1e-6) / 1e12, 2)
            d["hbm_frac"] = round(alg[key]["bytes"] / (us * 1e-6) / 1e9 / PEAK_HBM_GBS, 4)
        per_stage[n] = d

    if len(calls) == 1:
        workload = (f"config {args.config} / {shape.name}: T={shape.T}, {shape.d_in}->{shape.d_out}, N={shape.N}, "
                    f"r={shape.r}, top-{shape.k}, s={shape.scale}, {shape.routing} routing")
    else:
        workload = (f"config {args.config}, all {len(calls)} layers per step (" +
                    ", ".join(f"{sh.name} {sh.d_in}->{sh.d_out}" for sh, *_ in calls) +
                    f"): T={shape.T}, N={shape.N}, r={shape.r}, top-{shape.k}")
    res = {
        "metric": "MeteoRA-layer tokens/s at Llama3-8B shapes (28 LoRAs, top-2); % HBM/MFMA peak",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": workload,
                   "inputs_resident_in_hbm": True,
                   "weights": "W_gate, A, B packed once before the timed region (meteora_pack_weights)"},
        "per_call_packing": {"ms_per_step": elapsed_repack * 1e3 / args.steps,
                             "value": shape.T * args.steps / elapsed_repack, "unit": "tokens/s",
                             "note": "same loop through meteora_linear_forward, which repacks W_gate, A, B "
                                     "into the workspace on every call"},
        "roofline": roofline,
        "stages": per_stage,
    }
    if graph_ms is not None:
        res["hip_graph"] = {"ms_per_step": graph_ms, "value": shape.T / (graph_ms * 1e-3), "unit": "tokens/s",
                            "note": "the same step replayed from one captured HIP graph"}
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(shape, ops)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
