"""The paper's own forward-pass variants of the MeteoRA layer, timed on the same MI355X beside this library.

Sec. 3.3 describes three PyTorch-level ways to evaluate Eq. 2 and App. A.7 times them on random
pseudo data; they are rebuilt here from those descriptions with plain PyTorch-ROCm ops (rocBLAS /
hipBLASLt underneath) as measured context, on the same seeded synthetic workload as bench.py:

  single-lora    the upper bound: every token uses one adapter, no gate (base GEMM + one LoRA)
  loop-original  for each adapter i: gather the tokens routed to it, ((X_i A_i) B_i), scatter-add
  bmm-torch      gather A, B per (token, slot) pair (T*k/N times the adapter memory), two bmm,
                 weighted sum (Eq. 5)

Each variant's output is also compared with this library's (max |diff| / max |y|): they round
intermediates to bf16, so they agree to bf16 accuracy, not bit for bit.  One JSON line is printed.

    python bench_variants.py [--config 2] [--layer 0] [--steps 50] [--warmup 10]
"""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--layer", type=int, default=0)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    args = ap.parse_args()

    import torch
    import torch.nn.functional as F
    import paper_2405_13053_amd as m
    from gen import inputs as gen

    torch.cuda.set_device(0)
    seed, layers = gen.config_layers(args.config)
    shape = layers[args.layer]
    if shape.dtype != "bf16":
        sys.exit("bench_variants.py: bf16 configurations only")
    ops = gen.make_layer(shape, seed, args.layer)
    dt = torch.bfloat16
    x, W, A, B = (torch.from_numpy(ops[n]).cuda().to(dt) for n in ("x", "W", "A", "B"))
    Wg = torch.from_numpy(ops["W_gate"]).cuda()
    bias = None if ops["bias"] is None else torch.from_numpy(ops["bias"]).cuda()
    T, N, k, r, s = shape.T, shape.N, shape.k, shape.r, shape.scale

    ws = torch.empty(m.workspace_bytes(T, shape.d_in, shape.d_out, N, r, k, dt), dtype=torch.uint8, device="cuda")
    packed = m.pack_weights(Wg, A, B)
    out = torch.empty((T, shape.d_out), dtype=dt, device="cuda")

    def gate():   # fp32 gate, top-k, softmax over the k selected (Eq. 3)
        g = x.float() @ Wg
        if bias is not None:
            g = g + bias
        top, idx = torch.topk(g, k, dim=1)
        return idx, torch.softmax(top, dim=1)

    def this_library():
        return m.linear_forward(x, W, Wg, bias, A, B, k, s, out=out, ws=ws, packed=packed)

    def base_only():
        return F.linear(x, W)

    def single_lora():
        return F.linear(x, W) + s * ((x @ A[0]) @ B[0])

    def loop_original():
        idx, w = gate()
        y = F.linear(x, W)
        for i in range(N):
            tok, slot = torch.nonzero(idx == i, as_tuple=True)
            if tok.numel() == 0:
                continue
            delta = (x[tok] @ A[i]) @ B[i]
            y.index_add_(0, tok, (s * w[tok, slot]).to(dt).unsqueeze(1) * delta)
        return y

    def bmm_torch():
        idx, w = gate()
        flat = idx.reshape(-1)
        Ag, Bg = A[flat], B[flat]                                   # [T*k, d_in, r], [T*k, r, d_out]
        xs = x.repeat_interleave(k, dim=0).unsqueeze(1)              # [T*k, 1, d_in]
        delta = torch.bmm(torch.bmm(xs, Ag), Bg).reshape(T, k, -1)   # [T, k, d_out]
        return F.linear(x, W) + s * (w.to(dt).unsqueeze(2) * delta).sum(dim=1)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / args.steps

    ref = this_library().float()
    scale_ref = float(ref.abs().max())
    res = {"workload": f"config {args.config} / {shape.name}: T={T}, {shape.d_in}->{shape.d_out}, N={N}, r={r}, "
                       f"top-{k}, {shape.routing} routing", "steps": args.steps, "variants": {}}
    pair_mem = T * k * (shape.d_in * r + r * shape.d_out) * 2
    variants = [("this_library", this_library), ("base_gemm_only_torch", base_only), ("single_lora_torch", single_lora),
                ("loop_original_torch", loop_original)]
    if pair_mem < 64 << 30:
        variants.append(("bmm_torch", bmm_torch))
    # bring the clocks and caches to a steady state first: whatever is timed first would otherwise pay for it
    for _ in range(3):
        for _, fn in variants[:3]:
            for _ in range(10):
                fn()
    torch.cuda.synchronize()
    for name, fn in variants:
        us = timed(fn)
        d = {"us": round(us, 1), "tokens_per_s": round(T / (us * 1e-6))}
        if name in ("loop_original_torch", "bmm_torch"):
            d["max_rel_diff_vs_this_library"] = float((fn().float() - ref).abs().max()) / scale_ref
        if name == "bmm_torch":
            d["gathered_adapter_bytes"] = pair_mem
        res["variants"][name] = d
    v = res["variants"]
    res["ratios"] = {"loop_original / this_library": round(v["loop_original_torch"]["us"] / v["this_library"]["us"], 2),
                     "this_library / single_lora": round(v["this_library"]["us"] / v["single_lora_torch"]["us"], 2)}
    if "bmm_torch" in v:
        res["ratios"]["loop_original / bmm_torch"] = round(v["loop_original_torch"]["us"] / v["bmm_torch"]["us"], 2)
        res["ratios"]["bmm_torch / this_library"] = round(v["bmm_torch"]["us"] / v["this_library"]["us"], 2)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
