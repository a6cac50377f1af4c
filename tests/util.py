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


def sample_rows(T, counts=None, offsets=None, bucket_tok=None, n_strided=256, n_extreme=8, block=128):
    """Deterministic row sample: at least 256 evenly strided rows, one row in every block of `block` rows (at an
    offset inside the block that changes from block to block, so that every row tile of a GEMM and different
    positions inside the tiles are compared), plus rows of the smallest non-empty and the largest bucket."""
    n_strided = max(n_strided, 256)
    rows = set(np.linspace(0, T - 1, min(T, n_strided)).astype(np.int64).tolist())
    for b in range((T + block - 1) // block):
        lo, hi = b * block, min(T, (b + 1) * block)
        rows.add(lo + (b * 37 + 11) % (hi - lo))
    rows.add(T - 1)
    if counts is not None:
        nz = np.nonzero(counts)[0]
        if nz.size:
            small = nz[np.argmin(counts[nz])]
            large = int(np.argmax(counts))
            for j in (small, large):
                rows.update(bucket_tok[offsets[j]:offsets[j + 1]][:n_extreme].tolist())
    return np.array(sorted(rows), dtype=np.int32)


def weight_bound(ops, idx_ref, inv_temperature=1.0):
    """Per-token bound on |w_gpu - w_oracle| of the Eq. 3 weights, [T, 1].

    1e-6 for the softmax arithmetic itself (exp and division in fp32), plus the effect of the fp32 summation noise
    of the logits: sum_j |d w_i / d g_j| = 2 w_i (1 - w_i) <= 1/2, and the noise of a selected logit is bounded, as
    the gate test requires of the kernel's logits, by 8 * 2^-24 * (sum_i |x_i * W_gate_ij| + |bias_j|); a
    temperature scales the logit differences, and with them the noise, by 1/tau."""
    mag = np.abs(ops["x"].astype(np.float64)) @ np.abs(ops["W_gate"].astype(np.float64))
    if ops["bias"] is not None:
        mag = mag + np.abs(ops["bias"].astype(np.float64))
    noise = 8 * 2.0 ** -24 * np.take_along_axis(mag, idx_ref.astype(np.int64), axis=1).max(axis=1, keepdims=True)
    return 1e-6 + 0.5 * abs(inv_temperature) * noise


def oracle_routing(ops, k):
    """Oracle logits (fp32), top-k and weights for all tokens, and the buckets."""
    g64 = oracle.gate_logits(ops["x"], ops["W_gate"], ops["bias"])
    g32 = g64.astype(np.float32)
    idx, w = oracle.topk_softmax(g32, k)
    return g64, g32, idx, w
