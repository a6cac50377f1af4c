"""Base projection of the layer beside the vendor GEMM, on the same operands, on one MI355X.

Times, alternately and with hipEvents, on the x and W of a seeded configuration:

  meteora_base_gemm      this library's bf16 MFMA kernel, no LoRA extension (2*T*d_in*d_out flop)
  meteora layer GEMM     the same kernel inside meteora_linear_forward_packed (stage `gemm`: with the fused expand)
  vendor                 torch.matmul(x, W^T), i.e. the hipBLASLt kernel PyTorch-ROCm picks

The vendor kernel is measured context for the matrix-core ceiling discussion: it is not part of the library and
no library path calls it.  Run under `rocprofv3 --pmc ...` the same command gives both kernels' counters side by
side (profiles/gemm_vs_vendor_config2.md).  Prints one JSON line.

    python bench_gemm.py [--config 2] [--layer 0] [--iters 200] [--rounds 5] [--sample-clock]

--sample-clock reads the driver's sysfs files for the current shader clock (pp_dpm_sclk) and the socket power
(hwmon power1_input) from a host thread about every half millisecond while each timed block runs, and reports
their medians per kernel: the two GEMMs draw the same power, at the board's limit, at different clocks.
"""
import argparse
import glob
import json
import os
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--layer", type=int, default=0)
    ap.add_argument("--iters", type=int, default=200, help="launches per timed block")
    ap.add_argument("--rounds", type=int, default=5, help="alternations between the kernels")
    ap.add_argument("--sample-clock", action="store_true",
                    help="sample shader clock and socket power from sysfs during the timed blocks")
    args = ap.parse_args()

    import torch
    import paper_2405_13053_amd as m
    from gen import inputs as gen

    torch.cuda.set_device(0)
    seed, layers = gen.config_layers(args.config)
    sh = layers[args.layer]
    if sh.dtype != "bf16":
        sys.exit("bench_gemm.py: bf16 configurations only")
    ops = gen.make_layer(sh, seed, args.layer)
    dt = torch.bfloat16
    x, W, A, B = (torch.from_numpy(ops[n]).cuda().to(dt) for n in ("x", "W", "A", "B"))
    Wg = torch.from_numpy(ops["W_gate"]).cuda()
    bias = None if ops["bias"] is None else torch.from_numpy(ops["bias"]).cuda()
    out = torch.empty((sh.T, sh.d_out), dtype=dt, device="cuda")
    out_v = torch.empty_like(out)
    ws = torch.empty(m.workspace_bytes(sh.T, sh.d_in, sh.d_out, sh.N, sh.r, sh.k, dt), dtype=torch.uint8, device="cuda")
    packed = m.pack_weights(Wg, A, B)

    def ours():
        m.base_gemm(x, W, out=out)

    def vendor():
        torch.matmul(x, W.t(), out=out_v)

    def layer():
        m.linear_forward(x, W, Wg, bias, A, B, sh.k, sh.scale, out=out, ws=ws, packed=packed)

    sclk_files = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))[:1]
    power_files = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"))[:1]
    samples = {}   # kernel name -> list of (sclk MHz, power W)

    def sample_loop(stop, acc):
        while not stop.is_set():
            mhz = watts = None
            try:
                star = [ln for ln in open(sclk_files[0]).read().splitlines() if "*" in ln][0]
                mhz = int(star.split(":")[1].lower().split("mhz")[0])
            except (IndexError, OSError, ValueError):
                pass
            try:
                watts = int(open(power_files[0]).read()) / 1e6
            except (IndexError, OSError, ValueError):
                pass
            acc.append((mhz, watts))
            time.sleep(0.0005)

    def timed(fn, n, name=None):
        stop, th = threading.Event(), None
        if args.sample_clock and name is not None:
            th = threading.Thread(target=sample_loop, args=(stop, samples.setdefault(name, [])))
            th.start()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        if th is not None:
            stop.set()
            th.join()
        return e0.elapsed_time(e1) * 1e3 / n

    for fn in (ours, vendor, layer):
        for _ in range(20):
            fn()
    torch.cuda.synchronize()
    res = {"ours_base_gemm_us": [], "vendor_us": [], "layer_call_us": []}
    for _ in range(args.rounds):
        res["ours_base_gemm_us"].append(round(timed(ours, args.iters, "ours_base_gemm"), 2))
        res["vendor_us"].append(round(timed(vendor, args.iters, "vendor"), 2))
        res["layer_call_us"].append(round(timed(layer, args.iters, "layer_call"), 2))
    # the layer's own GEMM launch (with the fused expand), from the library's stage events
    m.stage_timing_enable(True)
    for _ in range(100):
        layer()
    torch.cuda.synchronize()
    stages, _ = m.stage_timing_read()
    m.stage_timing_enable(False)
    gemm_stage_us = stages["gemm"][0] * 1e3 / max(stages["gemm"][1], 1)
    flop = 2.0 * sh.T * sh.d_in * sh.d_out
    best = lambda v: min(v)
    rel = float((out_v.float() - (m.base_gemm(x, W)).float()).abs().max() / out_v.float().abs().max())
    def median(v):
        v = sorted(x for x in v if x is not None)
        return v[len(v) // 2] if v else None

    # the first block of a kernel still runs at the clock the previous kernel left: medians over the later samples
    clock = {name: {"sclk_MHz": median([a for a, _ in acc[len(acc) // 3:]]),
                    "power_W": median([b for _, b in acc[len(acc) // 3:]]), "samples": len(acc)}
             for name, acc in samples.items()}
    print(json.dumps({
        "workload": f"config {args.config} / {sh.name}: T={sh.T}, {sh.d_in}->{sh.d_out}, bf16",
        "iters_per_block": args.iters, "rounds": args.rounds, **res,
        "layer_gemm_stage_us": round(gemm_stage_us, 2),
        "TFLOP/s": {"ours_base_gemm": round(flop / best(res["ours_base_gemm_us"]) / 1e6, 1),
                    "vendor": round(flop / best(res["vendor_us"]) / 1e6, 1),
                    "layer_gemm_stage (base + expand flops)": round(
                        (flop + 2.0 * sh.T * sh.k * sh.r * sh.d_out) / gemm_stage_us / 1e6, 1)},
        "max_rel_diff_ours_vs_vendor": rel,
        **({"sampled_clock_and_power": clock} if args.sample_clock else {}),
        "note": "timed blocks run one kernel back to back: under sustained matrix-core load the chip clocks lower "
                "than inside the layer call, where lighter kernels sit between two GEMMs"}))


if __name__ == "__main__":
    main()
