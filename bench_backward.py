"""Gate-training step of one MeteoRA module on one MI355X: forward (Eq. 2) + gate gradients (Sec. 3.2, Eq. 4).

Workload: the layer of bench.py's headline configuration (T = 4096 tokens, 4096 -> 4096, N = 28 adapters of
rank 8, top-2, bf16, seeded synthetic values), with an upstream gradient dy and per-token task labels from
gen.inputs.make_training_signals.  Times meteora_gate_backward alone and together with the forward call whose
routing and products of x it reuses, without and with the module's input gradient dx (one more GEMM of the
forward's size), with HIP events on the launch stream, inputs resident in HBM.  Prints one JSON line; the
oracle's rate on a bounded token sample is reported beside it (a baseline, not a target).

    python bench_backward.py [--steps 200] [--warmup 20] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--beta", type=float, default=0.25)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()

    import numpy as np
    import torch
    import paper_2405_13053_amd as m
    from gen import inputs as gen

    torch.cuda.set_device(0)
    seed, shapes = gen.config_layers(2)
    s = shapes[0]
    ops = gen.make_layer(s, seed)
    dy, labels = gen.make_training_signals(s, seed)
    bf = torch.bfloat16
    dev = {n: torch.from_numpy(ops[n]).cuda().to(bf) for n in ("x", "W", "A", "B")}
    Wg = torch.from_numpy(ops["W_gate"]).cuda()
    dyd = torch.from_numpy(dy).cuda().to(bf)
    lab = torch.from_numpy(labels).cuda()
    packed = m.pack_weights(Wg, dev["A"], dev["B"])
    out = torch.empty((s.T, s.d_out), dtype=bf, device="cuda")
    ws_f = torch.empty(m.workspace_bytes(s.T, s.d_in, s.d_out, s.N, s.r, s.k, bf), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(m.gate_backward_workspace_bytes(s.T, s.d_in, s.d_out, s.N, s.r, s.k, bf), dtype=torch.uint8,
                       device="cuda")

    W_t = dev["W"].t().contiguous()   # the frozen base weight in the orientation the input gradient streams

    def backward(idx=None, w=None, forward_ws=None, dx=False):
        return m.gate_backward(dev["x"], dyd, None, dev["B"], packed, s.k, s.scale, labels=lab, beta=args.beta,
                               topk_idx=idx, topk_w=w, ws=ws_b, forward_ws=forward_ws, A=dev["A"], W_gate=Wg,
                               W_t=W_t, want_dx=dx)

    def forward():
        return m.linear_forward(dev["x"], dev["W"], Wg, None, dev["A"], dev["B"], s.k, s.scale, out=out, ws=ws_f,
                                return_routing=True, packed=packed)

    def both():
        _, idx, w = forward()
        backward(idx, w, ws_f)   # the forward call's products of x are read, not computed again

    def both_dx():
        _, idx, w = forward()
        backward(idx, w, ws_f, dx=True)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        st = torch.cuda.current_stream()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(st)
        for _ in range(args.steps):
            fn()
        e1.record(st)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps * 1e-3

    t_fwd = timed(forward)
    t_bwd = timed(backward)
    t_both = timed(both)
    t_bwd_dx = timed(lambda: backward(dx=True))
    t_both_dx = timed(both_dx)

    # HBM bytes one backward call has to move: x twice (products, x^T d_logits), dy, Wcat, B, the fp32 K-split
    # partials written and read back (all of the gate columns, the selected adapters' r columns), the padded
    # logit gradients, the slice partials of dW_gate written and read, dW_gate.
    T, d_in, d_out, N, r, k = s.T, s.d_in, s.d_out, s.N, s.r, s.k
    CR, NR = 96 + N * r, N * r
    need = ws_b.numel()
    algorithmic = (2 * T * d_in * 2 + T * d_out * 2 + CR * d_in * 2 + NR * d_out * 2 + d_in * N * 4)
    res = {
        "metric": "gate-training step of one MeteoRA module (tokens/s)",
        "config": {"workload": f"T={T} tokens, {d_in}->{d_out}, N={N}, r={r}, top-{k}, bf16, beta={args.beta}; "
                               "forward = meteora_linear_forward_packed, backward = meteora_gate_backward"},
        "backward": {"us_per_call": t_bwd * 1e6, "tokens_per_s": T / t_bwd,
                     "input_GB/s": algorithmic / t_bwd / 1e9, "input_bytes": algorithmic,
                     "workspace_bytes": need},
        "backward_with_dx": {"us_per_call": t_bwd_dx * 1e6, "tokens_per_s": T / t_bwd_dx,
                             "PFLOP/s_of_dx_gemm_equivalent": 2.0 * T * d_in * d_out / t_bwd_dx / 1e15},
        "forward": {"us_per_call": t_fwd * 1e6},
        "forward_plus_backward": {"us_per_call": t_both * 1e6, "tokens_per_s": T / t_both},
        "forward_plus_backward_with_dx": {"us_per_call": t_both_dx * 1e6, "tokens_per_s": T / t_both_dx},
        "steps": args.steps, "warmup": args.warmup, "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
    }
    if not args.no_cpu_baseline:
        from oracle import gate_backward as ob
        import oracle
        n = 256
        t0 = time.perf_counter()
        ob.gate_backward(ops["x"][:n], dy[:n], ops["W_gate"], None, ops["A"], ops["B"], k, s.scale, labels[:n], args.beta)
        dt = time.perf_counter() - t0
        res["cpu_baseline"] = {"value": n / dt, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"first {n} tokens of the same layer, oracle/gate_backward.py"}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
