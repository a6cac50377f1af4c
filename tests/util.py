"""Helpers shared by the GPU parity tests (no layer arithmetic here)."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from gen import inputs as gen
from oracle import margin


def torch_dtype(shape):
    return torch.bfloat16 if shape.dtype == "bf16" else torch.float32


def to_dev(a, dtype):
    """float32 numpy array (values exact in `dtype`) -> device tensor of that dtype."""
    if a is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda").to(dtype)


def make_case(shape, seed, layer=0, condition=True):
    """Draw a layer's operands (margin-conditioned x) and their device copies."""
    ops = gen.make_layer(shape, seed, layer)
    if condition:
        margin.condition_margins(shape, seed, layer, ops["x"], ops["W_gate"], ops["bias"], 1e-3)
    dt = torch_dtype(shape)
    dev = {n: to_dev(ops[n], dt) for n in ("x", "W", "A", "B")}
    dev["W_gate"] = to_dev(ops["W_gate"], torch.float32)
    dev["bias"] = to_dev(ops["bias"], torch.float32)
    return ops, dev


def rel_max_err(y_gpu: torch.Tensor, y_ref: np.ndarray) -> float:
    """max|y - y_ref| / max|y_ref| over the compared rows."""
    y = y_gpu.detach().to(torch.float64).cpu().numpy()
    return float(np.abs(y - y_ref).max() / np.abs(y_ref).max())


def tol(shape) -> float:
    """Output tolerance: 5e-3 for bf16 storage with fp32 accumulation, 1e-5 for fp32."""
    return 5e-3 if shape.dtype == "bf16" else 1e-5


def sample_rows(T, counts=None, offsets=None, bucket_tok=None, n_strided=256, n_extreme=8):
    """Deterministic row sample: strided rows plus rows of the smallest non-empty and largest bucket."""
    rows = set(np.linspace(0, T - 1, min(T, n_strided)).astype(np.int64).tolist())
    if counts is not None:
        nz = np.nonzero(counts)[0]
        if nz.size:
            small = nz[np.argmin(counts[nz])]
            large = int(np.argmax(counts))
            for j in (small, large):
                rows.update(bucket_tok[offsets[j]:offsets[j + 1]][:n_extreme].tolist())
    return np.array(sorted(rows), dtype=np.int32)


def oracle_routing(ops, k):
    """Oracle logits (fp32), top-k and weights for all tokens, and the buckets."""
    g64 = oracle.gate_logits(ops["x"], ops["W_gate"], ops["bias"])
    g32 = g64.astype(np.float32)
    idx, w = oracle.topk_softmax(g32, k)
    return g64, g32, idx, w
