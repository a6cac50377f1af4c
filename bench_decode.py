"""Decode step at model scale: every MeteoRA linear of a Llama3-8B-shaped model in one step.

The paper embeds the adapters in all seven linear layers of each of the 32 decoder blocks (224 MeteoRA
modules, Sec. 3.1 / Sec. 4.1) and measures generation speed (Sec. 4.3, App. A.7).  One decode step
pushes the current batch of tokens through all of them.  This script times exactly that part of a
step on one MI355X: 32 x (q, k, v, o, gate, up, down) layer calls with their own base weight, gate
and 28 rank-8 adapters each (seeded synthetic values; attention, norms and the residual stream are
not modelled, every layer gets an input of its own shape), so the 14 GB of base weights stream from
HBM once per step as in real decoding.  It reports the step eagerly enqueued (224 calls of
meteora_linear_forward_packed) and replayed from ONE captured HIP graph, which removes the host-side
launch cost when it dominates.  --group sends the layers of a block that share an input (q/k/v, gate/up)
through meteora_linear_forward_group, which runs each group in two launches.  Prints one JSON line.

    python bench_decode.py [--tokens 64] [--blocks 32] [--steps 20] [--warmup 3] [--group]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

D, KV, FFN = 4096, 1024, 14336
LAYERS = [("q_proj", D, D), ("k_proj", D, KV), ("v_proj", D, KV), ("o_proj", D, D),
          ("gate_proj", D, FFN), ("up_proj", D, FFN), ("down_proj", FFN, D)]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--tokens", type=int, default=64)
    ap.add_argument("--blocks", type=int, default=32)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--adapters", type=int, default=28)
    ap.add_argument("--rank", type=int, default=8)
    ap.add_argument("--topk", type=int, default=2)
    ap.add_argument("--group", action="store_true",
                    help="run the layers that share an input (q/k/v, gate/up) through meteora_linear_forward_group")
    args = ap.parse_args()

    import torch
    import paper_2405_13053_amd as m

    torch.cuda.set_device(0)
    dt = torch.bfloat16
    T, N, r, k, s = args.tokens, args.adapters, args.rank, args.topk, 2.0
    gen = torch.Generator(device="cuda").manual_seed(7)

    def randn(shape, std, dtype=dt):
        return (torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32) * std).to(dtype)

    xs = {d_in: randn((T, d_in), 1.0) for d_in in (D, FFN)}
    calls, weight_bytes = [], 0
    ws_bytes = 0
    groups = []   # per block: [q, k, v], [o], [gate, up], [down]
    for b in range(args.blocks):
        block = []
        for name, d_in, d_out in LAYERS:
            W = randn((d_out, d_in), d_in ** -0.5)
            Wg = randn((d_in, N), d_in ** -0.5, torch.float32)
            A = randn((N, d_in, r), d_in ** -0.5)
            B = randn((N, r, d_out), r ** -0.5)
            packed = m.pack_weights(Wg, A, B)
            out = torch.empty((T, d_out), dtype=dt, device="cuda")
            calls.append((xs[d_in], W, Wg, A, B, packed, out))
            block.append({"W": W, "W_gate": Wg, "gate_bias": None, "A": A, "B": B, "packed": packed, "out": out})
            weight_bytes += W.numel() * 2 + A.numel() * 2 + B.numel() * 2 + Wg.numel() * 4
            ws_bytes = max(ws_bytes, m.workspace_bytes(T, d_in, d_out, N, r, k, dt))
        for members, d_in in ((block[0:3], D), (block[3:4], D), (block[4:6], D), (block[6:7], FFN)):
            groups.append((xs[d_in], members))
            ws_bytes = max(ws_bytes, m.group_workspace_bytes([mb["W"].shape[0] for mb in members], T, d_in, N, r, k, dt))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")   # the calls of a step run one after the other
    torch.cuda.synchronize()

    def step_single():
        for x, W, Wg, A, B, packed, out in calls:
            m.linear_forward(x, W, Wg, None, A, B, k, s, out=out, ws=ws, packed=packed)

    def step_group():
        for x, members in groups:
            m.linear_forward_group(x, members, k, s, ws=ws)

    step = step_group if args.group else step_single

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / args.steps

    eager_s = timed(step)
    # host cost of enqueueing one step (no GPU wait inside the loop): the part a graph removes
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    step()
    enqueue_s = time.perf_counter() - t0
    torch.cuda.synchronize()

    ref = [c[-1].clone() for c in calls[:7]]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for c in calls[:7]:
        c[-1].fill_(float("nan"))
    graph.replay()
    torch.cuda.synchronize()
    same = all(torch.equal(c[-1], o) for c, o in zip(calls[:7], ref))
    graph_s = timed(graph.replay)

    n_layers = len(calls)
    res = {
        "metric": "decode step over all MeteoRA linears of a Llama3-8B-shaped model (tokens/s of the batch)",
        "config": {"workload": f"{args.blocks} blocks x 7 layers = {n_layers} MeteoRA layers per step, T={T} tokens, "
                               f"N={N}, r={r}, top-{k}, bf16, distinct weights per layer",
                   "weights_streamed_per_step_GB": round(weight_bytes / 1e9, 2),
                   "calls": "meteora_linear_forward_group on [q,k,v], [o], [gate,up], [down]" if args.group
                            else "meteora_linear_forward_packed per layer"},
        "eager": {"ms_per_step": eager_s * 1e3, "us_per_layer": eager_s * 1e6 / n_layers,
                  "tokens_per_s": T / eager_s, "host_enqueue_ms_per_step": enqueue_s * 1e3},
        "hip_graph": {"ms_per_step": graph_s * 1e3, "us_per_layer": graph_s * 1e6 / n_layers,
                      "tokens_per_s": T / graph_s, "replay_matches_eager_bit_for_bit": bool(same),
                      "GB/s_of_weights": weight_bytes / graph_s / 1e9},
        "steps": args.steps, "warmup": args.warmup, "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
    }
    print(json.dumps(res))


if __name__ == "__main__":
    main()
