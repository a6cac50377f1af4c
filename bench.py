"""Benchmark of the MeteoRA linear-layer forward on one MI355X.

A "step" is one call of the whole layer over one batch of the workload (all stages of the hot
path: gate, top-k, bucketing, shrink, base GEMM, expand).  The weights are static during inference,
so their kernel-side layouts are packed once before the timed region (meteora_pack_weights) and
every step calls meteora_linear_forward_packed; the same loop with per-call packing
(meteora_linear_forward) is timed as well and reported beside it.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--layer 0] [--tokens T]
                    [--no-cpu-baseline] [--no-extra-configs] [--graph] [--pmc-calibration]
    python bench.py --summarize-pmc FETCH_DIR WRITE_DIR [--summarize-workload configC/layerL]
                                                            (no GPU: writes profiles/hbm_traffic.json)

`value` is the headline workload: configuration 2 (q_proj-shaped prefill) unless --config/--layer say
otherwise.  When the headline is configuration 2, the line also carries, under `configs`, the other seeded
configurations that fit one GPU (3: gate/up and down projection; 4: both decode layers; 5: the seven
projections of a block per step), each with its own time per step, tokens/s and the roofline fraction of its
dominant kernel against the bound that applies to it (matrix cores for the prefill GEMMs, HBM for the
weight-streaming decode launch).  --no-extra-configs leaves them out (profiling runs).

The defaults (1000 timed steps after 100 warm-up steps, about 0.15 s) reach the steady state of the
clocks; runs of a few dozen steps measure 4-5% slower.  --graph also replays the step from a captured
HIP graph.  --tokens T runs the configuration's layer shapes with T tokens instead of its own batch.
--layer -1 runs every layer of the configuration one after the other per step.

Per-stage durations come from hipEvents that the library records around each stage on the launch stream; a
reading is the stage's kernels plus the dispatch gap in front of them (about 2 us per launch more than rocprofv3's
kernel trace shows for the same dispatches, see profiles/), so the roofline fractions derived from them err low.

--pmc-calibration runs a plain device copy of known size (256 MiB, three times) before the workload, so that a
rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run of this command holds its own calibration of the counters' units;
--summarize-pmc reads the CSV files of two such runs and writes profiles/hbm_traffic.json, from which later runs
take `roofline.traffic`.
"""
import argparse
import csv
import glob
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
CALIBRATION_COPY_BYTES = 256 << 20
METRIC = "MeteoRA-layer tokens/s at Llama3-8B shapes (28 LoRAs, top-2); % HBM/MFMA peak"


def algorithmic(shape):
    """Algorithmic flops and bytes of each stage of one layer call (e = bytes per element)."""
    s = shape
    e = 2 if s.dtype == "bf16" else 4
    T, di, do, N, r, k = s.T, s.d_in, s.d_out, s.N, s.r, s.k
    touched = min(N, T * k)   # adapters a batch can touch at all
    return {
        "gate": {"flops": 2.0 * T * di * N, "bytes": T * di * e + di * N * 4 + T * k * 8},
        "shrink": {"flops": 2.0 * T * k * di * r, "bytes": T * di * e + N * di * r * e + T * k * r * 4},
        "expand": {"flops": 2.0 * T * k * r * do, "bytes": T * k * r * 4 + N * r * do * e + T * do * e},
        "gemm": {"flops": 2.0 * T * di * do, "bytes": T * di * e + di * do * e + T * do * e},
        # a fully fused layer's floor: every operand once (adapters: those the batch can touch)
        "layer": {"flops": 2.0 * T * (di * do + di * N + k * r * (di + do)),
                  "bytes": T * di * e + di * do * e + di * N * 4 + touched * r * (di + do) * e + T * do * e},
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


def measured_traffic(config, layer):
    """HBM bytes per launch of the workload's dominant kernel from the tracked rocprofv3 summary, or None."""
    try:
        with open(TRAFFIC_FILE) as f:
            data = json.load(f)
    except (OSError, ValueError):
        return None, None
    ent = data.get("workloads", {}).get(f"config{config}/layer{layer}")
    if not ent:
        return None, None
    return ent.get("dominant_kernel_bytes"), {"file": "profiles/hbm_traffic.json", "kernel": ent.get("dominant_kernel"),
                                              "measured_at_head": ent.get("measured_at_head", data.get("head"))}


class Workload:
    """The layers of one configuration, resident on the GPU, with packed weights and workspaces."""

    def __init__(self, config, layer, tokens=0):
        import dataclasses
        import torch
        import paper_2405_13053_amd as m
        from gen import inputs as gen
        self.config, self.layer = config, layer
        seed, layers = gen.config_layers(config)
        if tokens > 0:
            layers = [dataclasses.replace(sh, T=tokens) for sh in layers]
        which = list(range(len(layers))) if layer < 0 else [layer]
        self.calls = []
        self.first_ops = None
        for li in which:
            sh = layers[li]
            ops_l = gen.make_layer(sh, seed, li)
            dt = torch.bfloat16 if sh.dtype == "bf16" else torch.float32
            dev = {n: torch.from_numpy(ops_l[n]).cuda().to(dt) for n in ("x", "W", "A", "B")}
            Wg = torch.from_numpy(ops_l["W_gate"]).cuda()
            bias = None if ops_l["bias"] is None else torch.from_numpy(ops_l["bias"]).cuda()
            out = torch.empty((sh.T, sh.d_out), dtype=dt, device="cuda")
            ws = torch.empty(m.workspace_bytes(sh.T, sh.d_in, sh.d_out, sh.N, sh.r, sh.k, dt), dtype=torch.uint8,
                             device="cuda")
            packed = m.pack_weights(Wg, dev["A"], dev["B"])   # once per set of adapters, outside the timed region
            self.calls.append((sh, dev, Wg, bias, out, ws, packed))
            if self.first_ops is None:
                self.first_ops = ops_l   # the CPU baseline samples the first layer
        self.shape = self.calls[0][0]
        self.m = m
        self.torch = torch

    def step(self):
        for sh, dev, Wg, bias, out, ws, packed in self.calls:
            self.m.linear_forward(dev["x"], dev["W"], Wg, bias, dev["A"], dev["B"], sh.k, sh.scale, out=out, ws=ws,
                                  packed=packed)

    def step_repack(self):
        for sh, dev, Wg, bias, out, ws, packed in self.calls:
            self.m.linear_forward(dev["x"], dev["W"], Wg, bias, dev["A"], dev["B"], sh.k, sh.scale, out=out, ws=ws)

    def timed(self, fn, steps, warmup):
        """Seconds for `steps` calls after `warmup` untimed ones: synchronised on both sides, the interval itself
        taken with events on the stream the calls are enqueued on (a host clock would add the wake-up after the
        final synchronisation, 2-3% of a 20-step run of this layer)."""
        torch = self.torch
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3

    def describe(self):
        shape = self.shape
        if len(self.calls) == 1:
            return (f"config {self.config} / {shape.name}: T={shape.T}, {shape.d_in}->{shape.d_out}, N={shape.N}, "
                    f"r={shape.r}, top-{shape.k}, s={shape.scale}, {shape.routing} routing")
        return (f"config {self.config}, all {len(self.calls)} layers per step (" +
                ", ".join(f"{sh.name} {sh.d_in}->{sh.d_out}" for sh, *_ in self.calls) +
                f"): T={shape.T}, N={shape.N}, r={shape.r}, top-{shape.k}")

    def stages(self, n_prof):
        """Per-stage microseconds per step from the library's own hipEvents (summed over the layers of the set)."""
        m, torch = self.m, self.torch
        m.stage_timing_enable(True)
        n_prof = max(1, min(n_prof, 200 // len(self.calls)))
        # first windows that are read and dropped, at least 5 ms of them: the events' own first use, and the clocks
        # after the pause that switching the timing on makes (a few thousand events are created), stay out of the
        # window that is reported
        t0 = time.perf_counter()
        while True:
            for _ in range(max(3, min(n_prof, 10))):
                self.step()
            m.stage_timing_read()
            if time.perf_counter() - t0 > 5e-3:
                break
        for _ in range(n_prof):
            self.step()
        torch.cuda.synchronize()
        stages, _ = m.stage_timing_read()
        m.stage_timing_enable(False)
        us = {n: ms * 1e3 / n_prof for n, (ms, c) in stages.items() if c > 0}
        launches = {n: c / n_prof for n, (ms, c) in stages.items() if c > 0}
        return us, launches

    def report(self, steps, warmup, repack=True, graph=False):
        """Time the workload and derive the per-stage and roofline figures."""
        torch = self.torch
        shape = self.shape
        res = {}
        # about 20 ms of untimed steps first: the shader clock comes up from idle over some 10 ms of work, and a short
        # run would otherwise time its first loop on the ramp
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < 20e-3:
            for _ in range(4):
                self.step()
            torch.cuda.synchronize()
        elapsed_repack = self.timed(self.step_repack, steps, warmup) if repack else None
        for _ in range(warmup):   # first launches (code loading) stay out of the stage readings
            self.step()
        # stage timing first, the headline loop last: the shader clock takes some 10 ms of work to come up from idle
        # (a 20-step loop timed 3 ms into the process read 148 us per step where the same loop read 127 later on)
        stage_us, launches = self.stages(steps)
        elapsed = self.timed(self.step, steps, warmup)
        graph_ms = None
        if graph:
            # the library allocates nothing and records no memset, so a step can be captured once and replayed
            side = torch.cuda.Stream()
            g = torch.cuda.CUDAGraph()
            torch.cuda.synchronize()
            with torch.cuda.stream(side):
                with torch.cuda.graph(g, stream=side):
                    self.step()
            graph_ms = self.timed(g.replay, steps, warmup) * 1e3 / steps
        res["ms_per_step"] = elapsed * 1e3 / steps
        res["value"] = shape.T * steps / elapsed

        alg = {}
        for sh, *_ in self.calls:
            for key, d in algorithmic(sh).items():
                acc = alg.setdefault(key, {"flops": 0.0, "bytes": 0.0})
                acc["flops"] += d["flops"]
                acc["bytes"] += d["bytes"]
        kernel_us = stage_us
        decode = "gate_logits" not in stage_us and "bucket" not in stage_us and "shrink" in stage_us and shape.T <= 64
        gemm_us = kernel_us["gemm"]
        if decode:
            # weight streaming: the launch that reads W (with the routing products riding in it) against HBM
            achieved = alg["gemm"]["bytes"] / (gemm_us * 1e-6) / 1e9
            traffic, source = (None, None) if len(self.calls) > 1 else measured_traffic(self.config, self.layer)
            roofline = {"kernel": "split-K base projection (streams W once; gate logits and every adapter's shrink in the same launch)",
                        "bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": achieved / PEAK_HBM_GBS, "traffic": traffic,
                        "algorithmic_bytes": alg["gemm"]["bytes"], "us": gemm_us,
                        "whole_call": {"algorithmic_bytes": alg["layer"]["bytes"],
                                       "GB/s": alg["layer"]["bytes"] / (res["ms_per_step"] * 1e-3) / 1e9,
                                       "frac": alg["layer"]["bytes"] / (res["ms_per_step"] * 1e-3) / 1e9 / PEAK_HBM_GBS}}
            if source:
                roofline["traffic_source"] = source
        else:
            gemm_flops = alg["gemm"]["flops"] + (alg["expand"]["flops"] if "expand" not in stage_us else 0.0)
            achieved = gemm_flops / (gemm_us * 1e-6) / 1e12
            traffic, source = (None, None) if len(self.calls) > 1 else measured_traffic(self.config, self.layer)
            roofline = {"kernel": "base GEMM (bf16 MFMA) with the LoRA expand fused" if shape.dtype == "bf16"
                        else "base GEMM (fp32)",
                        "bound": "mfma", "achieved": achieved, "peak": PEAK_MFMA_BF16_TFLOPS, "unit": "TFLOP/s",
                        "frac": achieved / PEAK_MFMA_BF16_TFLOPS, "traffic": traffic,
                        "algorithmic_bytes": alg["gemm"]["bytes"], "us": gemm_us}
            if source:
                roofline["traffic_source"] = source
        per_stage = {}
        # mid-sized batches: one launch computes the gate logits and the shrink (no bucket / shrink stage is timed);
        # its algorithmic work is the gate's plus the selected adapters' shrink, with x read once
        dense_route = "shrink" not in stage_us and "gate_logits" in stage_us
        if dense_route:
            alg["gate+shrink"] = {"flops": alg["gate"]["flops"] + alg["shrink"]["flops"],
                                  "bytes": alg["gate"]["bytes"] + alg["shrink"]["bytes"] -
                                           sum(sh.T * sh.d_in * (2 if sh.dtype == "bf16" else 4)
                                               for sh, *_ in self.calls)}
        for n, us in stage_us.items():
            key = {"gate_logits": "gate+shrink" if dense_route else "gate", "gate_topk": None, "bucket": None}.get(n, n)
            if decode:
                key = {"gemm": "gemm"}.get(n)
            d = {"us": round(us, 2)}
            if n == "gate_logits" and dense_route:
                d["covers"] = "gate logits and LoRA shrink in one launch; gate_topk = top-k, softmax and selection"
            if n == "shrink" and "gate_logits" not in stage_us and "bucket" not in stage_us:
                d["covers"] = "the tail launch: top-k, softmax, split-K reduction and LoRA expand"
            if key and key in alg:
                t = kernel_us[n] * 1e-6
                d["GB/s"] = round(alg[key]["bytes"] / t / 1e9, 1)
                d["TFLOP/s"] = round(alg[key]["flops"] / t / 1e12, 2)
                d["hbm_frac"] = round(alg[key]["bytes"] / t / 1e9 / PEAK_HBM_GBS, 4)
            per_stage[n] = d
        res["roofline"] = roofline
        res["stages"] = per_stage
        if elapsed_repack is not None:
            res["per_call_packing"] = {"ms_per_step": elapsed_repack * 1e3 / steps,
                                       "value": shape.T * steps / elapsed_repack, "unit": "tokens/s",
                                       "note": "same loop through meteora_linear_forward, which repacks W_gate, A, B "
                                               "into the workspace on every call"}
        if graph_ms is not None:
            res["hip_graph"] = {"ms_per_step": graph_ms, "value": shape.T / (graph_ms * 1e-3), "unit": "tokens/s",
                                "note": "the same step replayed from one captured HIP graph"}
        return res


def extra_configs(steps, warmup):
    """The other seeded configurations as entries of the same JSON line (bounded step counts)."""
    import torch
    out = {}
    plan = [("config3/gate_proj", 3, 0, "up_proj has the same shape and routing recipe"),
            ("config3/down_proj", 3, 2, None),
            ("config4/attn_proj", 4, 0, None),
            ("config4/mlp_up", 4, 1, None),
            ("config5/block", 5, -1, "the seven projections of a block, one call each per step")]
    for name, cfg, layer, note in plan:
        wl = Workload(cfg, layer)
        big = wl.shape.T > 64
        k = max(5, min(steps, 50 if big else 500))
        w = max(2, min(warmup, 10 if big else 50))
        r = wl.report(k, w, repack=False)
        ent = {"workload": wl.describe(), "steps": k, "warmup": w, "ms_per_step": r["ms_per_step"],
               "value": r["value"], "unit": "tokens/s", "roofline": r["roofline"], "stages": r["stages"]}
        if note:
            ent["note"] = note
        out[name] = ent
        del wl
        torch.cuda.empty_cache()
    return out


def paper_variants(wl, ms_layer, steps):
    """The paper's own schedules (Sec. 3.3) timed on the headline workload beside the layer call: loop-original and
    the gathered batched products through meteora_variant_forward, and the single-adapter upper bound (base GEMM +
    one LoRA for every token, no gate) composed from meteora_base_gemm and meteora_lora_forward."""
    torch, m = wl.torch, wl.m
    sh, dev, Wg, bias, out, ws, packed = wl.calls[0]
    dt = torch.bfloat16 if sh.dtype == "bf16" else torch.float32
    res = {"workload": wl.describe(), "this_library_us": round(ms_layer * 1e3, 1)}
    n = max(3, min(steps, 10))

    def timed(fn):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e6 / n

    for name, v in (("loop_original", m.LOOP_ORIGINAL), ("bmm_gather", m.BMM_GATHER)):
        need = m.variant_workspace_bytes(v, sh.T, sh.d_in, sh.d_out, sh.N, sh.r, sh.k, dt)
        vws = torch.empty(need, dtype=torch.uint8, device="cuda")
        us = timed(lambda: m.variant_forward(v, dev["x"], dev["W"], Wg, bias, dev["A"], dev["B"], sh.k, sh.scale,
                                             out=out, ws=vws))
        res[name] = {"us": round(us, 1), "workspace_bytes": need}
        del vws
        torch.cuda.empty_cache()
    # single-lora: every token through adapter 0 with weight 1
    idx0 = torch.zeros((sh.T, 1), dtype=torch.int32, device="cuda")
    w1 = torch.ones((sh.T, 1), dtype=torch.float32, device="cuda")
    A0, B0 = dev["A"][:1].contiguous(), dev["B"][:1].contiguous()
    lws = torch.empty(m.workspace_bytes(sh.T, sh.d_in, sh.d_out, 1, sh.r, 1, dt), dtype=torch.uint8, device="cuda")

    def single():
        m.base_gemm(dev["x"], dev["W"], out=out)
        m.lora_forward(dev["x"], A0, B0, idx0, w1, sh.scale, out=out, accumulate=True, ws=lws)
    res["single_lora"] = {"us": round(timed(single), 1)}
    lay = ms_layer * 1e3
    res["ratios"] = {"loop_original / single_lora": round(res["loop_original"]["us"] / res["single_lora"]["us"], 2),
                     "loop_original / bmm_gather": round(res["loop_original"]["us"] / res["bmm_gather"]["us"], 2),
                     "bmm_gather / single_lora": round(res["bmm_gather"]["us"] / res["single_lora"]["us"], 2),
                     "this_library / single_lora": round(lay / res["single_lora"]["us"], 2),
                     "loop_original / this_library": round(res["loop_original"]["us"] / lay, 2),
                     "bmm_gather / this_library": round(res["bmm_gather"]["us"] / lay, 2)}
    res["paper"] = ("on H800 (Sec. 3.3, Sec. 5, App. A.7): loop-original up to 10x single-lora; bmm-torch about 4x faster "
                    "than loop-original and about 2.5x slower than single-lora; its Triton kernel keeps about 80% of that")
    return res


def summarize_pmc(fetch_dir, write_dir, workload="config2/layer0"):
    """Read the counter CSVs of two rocprofv3 --pmc runs of `bench.py --pmc-calibration` (FETCH_SIZE, WRITE_SIZE)
    and write profiles/hbm_traffic.json: per kernel the average counter value per dispatch, the factor that turns it
    into KiB (from the known-size copy in the same run) and the resulting HBM bytes."""
    def read(d, counter):
        rows = {}
        for path in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
            with open(path, newline="") as f:
                for row in csv.DictReader(f):
                    if row["Counter_Name"] == counter:
                        rows.setdefault(row["Kernel_Name"], []).append(float(row["Counter_Value"]))
        return rows
    fetch, write = read(fetch_dir, "FETCH_SIZE"), read(write_dir, "WRITE_SIZE")
    if not fetch or not write:
        sys.exit("summarize-pmc: no FETCH_SIZE / WRITE_SIZE rows found")

    def copy_scale(rows):
        # the calibration copy: the runtime's device-to-device copy kernel, the first three dispatches of it are
        # --pmc-calibration's copies of CALIBRATION_COPY_BYTES each (they run before anything else)
        cand = [(k, v) for k, v in rows.items() if "copyBuffer" in k]
        if not cand or len(cand[0][1]) < 3:
            sys.exit("summarize-pmc: calibration copy kernel not found (run bench.py with --pmc-calibration)")
        name, vals = cand[0]
        avg = sum(vals[:3]) / 3.0
        return (CALIBRATION_COPY_BYTES / 1024.0) / avg, name, avg
    fs, fname, favg = copy_scale(fetch)
    wsc, wname, wavg = copy_scale(write)
    kernels = {}
    for k in sorted(set(fetch) | set(write)):
        if not ("meteora" in k or "gemm_mfma" in k or "route_" in k or "gate_" in k or "shrink_" in k or
                "bucket_" in k or "prep_kernel" in k):
            continue
        f, w = fetch.get(k, []), write.get(k, [])
        fa = sum(f) / len(f) if f else 0.0
        wa = sum(w) / len(w) if w else 0.0
        kernels[k] = {"dispatches": max(len(f), len(w)), "FETCH_SIZE_raw": fa, "WRITE_SIZE_raw": wa,
                      "read_bytes": fa * fs * 1024, "written_bytes": wa * wsc * 1024,
                      "bytes": (fa * fs + wa * wsc) * 1024}
    # the workload's dominant kernel: the 256 x 256 GEMM, else (decode) the split-K GEMM that streams W
    gemm = [k for k in kernels if "gemm_mfma_w3_kernel<4, 4" in k or "gemm_mfma_w3_kernel<4,4" in k]
    if not gemm:
        gemm = sorted((k for k in kernels if "gemm_mfma" in k), key=lambda k: -kernels[k]["bytes"])[:1]
    try:
        head = subprocess.check_output(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], text=True).strip()
    except Exception:
        head = None
    try:
        with open(TRAFFIC_FILE) as f:
            data = json.load(f)        # other workloads' entries are kept
    except (OSError, ValueError):
        data = {}
    data["command"] = ("rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE --output-format csv -d <dir> -o b -- python3 bench.py "
                       "[--config C --layer L] --steps 10 --warmup 3 --no-cpu-baseline --no-extra-configs "
                       "--pmc-calibration; then python3 bench.py --summarize-pmc <fetch dir> <write dir> "
                       "[--summarize-workload configC/layerL]")
    data.setdefault("workloads", {})[workload] = {
        "dominant_kernel": gemm[0] if gemm else None,
        "dominant_kernel_bytes": kernels[gemm[0]]["bytes"] if gemm else None,
        "measured_at_head": head,
        "calibration": {"copy_bytes": CALIBRATION_COPY_BYTES, "FETCH_SIZE_raw_for_copy": favg,
                        "WRITE_SIZE_raw_for_copy": wavg, "FETCH_SIZE_to_KiB": fs, "WRITE_SIZE_to_KiB": wsc,
                        "copy_kernel": fname[:80]},
        "kernels": kernels}
    if workload == "config2/layer0":
        data["head"] = head
        data["calibration"] = data["workloads"][workload]["calibration"]
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(data, f, indent=1)
        f.write("\n")
    print(json.dumps({"written": TRAFFIC_FILE, "workload": workload, "head": head,
                      "dominant_kernel": data["workloads"][workload]["dominant_kernel"],
                      "dominant_kernel_bytes": data["workloads"][workload]["dominant_kernel_bytes"]}))


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
    ap.add_argument("--no-extra-configs", action="store_true",
                    help="leave out the `configs` key (the other seeded configurations)")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step replayed from a captured HIP graph (reported as hip_graph)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="run a known-size device copy first (for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs)")
    ap.add_argument("--summarize-pmc", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"),
                    help="no GPU: turn two rocprofv3 --pmc output folders into profiles/hbm_traffic.json")
    ap.add_argument("--summarize-workload", default="config2/layer0", metavar="configC/layerL",
                    help="with --summarize-pmc: the workload the two runs profiled (its entry of the JSON is replaced)")
    args = ap.parse_args()
    if args.summarize_pmc:
        summarize_pmc(*args.summarize_pmc, workload=args.summarize_workload)
        return
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
                 "(the layer shards by tokens with no exchange step between the GPUs)")

    import torch
    torch.cuda.set_device(0)
    if args.pmc_calibration:
        a = torch.ones(CALIBRATION_COPY_BYTES // 4, dtype=torch.float32, device="cuda")
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    wl = Workload(args.config, args.layer, args.tokens)
    shape = wl.shape
    r = wl.report(args.steps, args.warmup, repack=True, graph=args.graph)
    res = {
        "metric": METRIC,
        "value": r["value"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": wl.describe(),
                   "inputs_resident_in_hbm": True,
                   "weights": "W_gate, A, B packed once before the timed region (meteora_pack_weights)"},
        "per_call_packing": r["per_call_packing"],
        "roofline": r["roofline"],
        "stages": r["stages"],
    }
    if "hip_graph" in r:
        res["hip_graph"] = r["hip_graph"]
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(shape, wl.first_ops)
    headline_default = args.config == 2 and args.layer == 0 and args.tokens == 0
    if headline_default and not args.no_extra_configs:
        res["paper_variants"] = paper_variants(wl, r["ms_per_step"], args.steps)
    del wl
    torch.cuda.empty_cache()
    if headline_default and not args.no_extra_configs:
        res["configs"] = extra_configs(args.steps, args.warmup)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
