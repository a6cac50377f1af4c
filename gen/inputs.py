"""Seeded synthetic inputs for the MeteoRA linear layer.

This module only draws random numbers and rounds them to the storage dtype.
It holds none of the layer's arithmetic (no gate, no top-k, no LoRA product),
so both the CPU oracle's tests and the HIP path's tests/benchmarks can share it.

Every tensor is an independent counter-based Philox stream keyed by
(seed, tensor tag, layer tag), so a tensor's values do not depend on the
order in which tensors are drawn, and one row of ``x`` can be re-drawn
without touching anything else.

Value distributions (all i.i.d. Gaussian; they stand in for the paper's
"randomly-generated pseudo data" efficiency experiment, App. A.7, at the
Llama3-8B / Llama2-13B layer shapes of Sec. 4.1):

    x       ~ N(0, 1)            [T, d_in]
    W       ~ N(0, 1/d_in)       [d_out, d_in]   (row-major, K-contiguous)
    W_gate  ~ N(0, 1/d_in)       [d_in, N]       (so logits are ~N(0,1))
    A_i     ~ N(0, 1/d_in)       [N, d_in, r]
    B_i     ~ N(0, 1/r)          [N, r, d_out]
    bias_j  = 2*ln(1/(j+1))      [N]             (only for "zipf" routing)

All arrays are returned as float32 numpy arrays.  For dtype "bf16" each
value of x, W, A, B is rounded once (round-to-nearest-even) to a value that
bfloat16 represents exactly; W_gate and bias always stay fp32.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional

import numpy as np

_TAGS = {"x": 1, "W": 2, "W_gate": 3, "A": 4, "B": 5, "dy": 6, "labels": 7}


@dataclasses.dataclass(frozen=True)
class LayerShape:
    """One MeteoRA linear layer's problem size (paper notation: T=b*s, n=N)."""

    T: int
    d_in: int
    d_out: int
    N: int
    r: int
    k: int
    scale: float = 2.0
    dtype: str = "bf16"          # "bf16" or "f32": storage type of x, W, A, B, out
    routing: str = "uniform"     # "uniform" (no bias) or "zipf" (bias 2*ln(1/(j+1)))
    name: str = ""


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even), keep fp32 storage."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def _stream(seed: int, tag: int, layer: int, redraw: int = 0) -> np.random.Generator:
    # Philox takes a 2x64-bit key; pack (seed, layer) and (tag, redraw) into it.
    key = [(seed & 0xFFFFFFFF) | ((layer & 0xFFFFFFFF) << 32),
           (tag & 0xFFFFFFFF) | ((redraw & 0xFFFFFFFF) << 32)]
    return np.random.Generator(np.random.Philox(key=key))


def _normal(seed, tag, layer, shape, std, dtype) -> np.ndarray:
    g = _stream(seed, tag, layer)
    a = g.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return round_to_bf16(a) if dtype == "bf16" else a


def zipf_bias(N: int) -> np.ndarray:
    """Gate bias b_j = 2*ln(1/(j+1)): makes adapter load Zipf-like."""
    j = np.arange(N, dtype=np.float64)
    return (2.0 * np.log(1.0 / (j + 1.0))).astype(np.float32)


def make_layer(shape: LayerShape, seed: int, layer: int = 0,
               only: Optional[tuple] = None) -> Dict[str, Optional[np.ndarray]]:
    """Draw all operands of one layer.  ``only`` restricts to a subset of names."""
    s = shape
    want = (lambda n: only is None or n in only)
    out: Dict[str, Optional[np.ndarray]] = {}
    if want("x"):
        out["x"] = _normal(seed, _TAGS["x"], layer, (s.T, s.d_in), 1.0, s.dtype)
    if want("W"):
        out["W"] = _normal(seed, _TAGS["W"], layer, (s.d_out, s.d_in),
                           1.0 / math.sqrt(s.d_in), s.dtype)
    if want("W_gate"):
        out["W_gate"] = _normal(seed, _TAGS["W_gate"], layer, (s.d_in, s.N),
                                1.0 / math.sqrt(s.d_in), "f32")
    if want("A"):
        out["A"] = _normal(seed, _TAGS["A"], layer, (s.N, s.d_in, s.r),
                           1.0 / math.sqrt(s.d_in), s.dtype)
    if want("B"):
        out["B"] = _normal(seed, _TAGS["B"], layer, (s.N, s.r, s.d_out),
                           1.0 / math.sqrt(s.r), s.dtype)
    if want("bias"):
        out["bias"] = zipf_bias(s.N) if s.routing == "zipf" else None
    return out


def redraw_rows(x: np.ndarray, rows: np.ndarray, shape: LayerShape, seed: int,
                layer: int, attempt: int) -> None:
    """Replace the given rows of ``x`` in place by fresh N(0,1) draws.

    Used by the tests' margin conditioning: a row whose gate logits are nearly
    tied is re-drawn from an independent stream keyed by (row, attempt), so the
    result is deterministic and independent of which other rows were re-drawn.
    """
    for t in np.asarray(rows, dtype=np.int64):
        g = _stream(seed, _TAGS["x"] | (int(t) + 1) << 8, layer, redraw=attempt)
        v = g.standard_normal(size=(shape.d_in,), dtype=np.float32)
        x[t, :] = round_to_bf16(v) if shape.dtype == "bf16" else v


def make_training_signals(shape: LayerShape, seed: int, layer: int = 0):
    """Inputs of a gate-training step on this layer (Sec. 3.2): the upstream gradient dy[T, d_out] ~ N(0, 1/d_out)
    in the storage dtype, and per-token task labels: tokens come in runs of 16 with one task each (a sample of
    the balanced training set is one task's), every 11th run unlabelled (-1)."""
    dy = _normal(seed, _TAGS["dy"], layer, (shape.T, shape.d_out), 1.0 / math.sqrt(shape.d_out), shape.dtype)
    runs = (shape.T + 15) // 16
    per_run = _stream(seed, _TAGS["labels"], layer).integers(0, shape.N, size=runs, dtype=np.int32)
    per_run[10::11] = -1
    labels = np.repeat(per_run, 16)[:shape.T].astype(np.int32)
    return dy, labels


# --------------------------------------------------------------------------
# The five seeded configurations.  Seed = config index - 1; config 1 is seed 0.
# Multi-layer configs draw each layer with its own ``layer`` tag.
# --------------------------------------------------------------------------

def config_layers(cfg: int):
    """Return (seed, [LayerShape, ...]) of configuration ``cfg`` in 1..5."""
    if cfg == 1:   # tiny fp32 layer
        return 0, [LayerShape(64, 256, 256, 4, 8, 2, 2.0, "f32", "uniform", "tiny")]
    if cfg == 2:   # Llama3-8B q_proj-shaped prefill
        return 1, [LayerShape(4096, 4096, 4096, 28, 8, 2, 2.0, "bf16", "uniform", "q_proj")]
    if cfg == 3:   # Llama3-8B MLP, Zipf-like adapter load
        return 2, [LayerShape(8192, 4096, 14336, 28, 8, 2, 2.0, "bf16", "zipf", "gate_proj"),
                   LayerShape(8192, 4096, 14336, 28, 8, 2, 2.0, "bf16", "zipf", "up_proj"),
                   LayerShape(8192, 14336, 4096, 28, 8, 2, 2.0, "bf16", "zipf", "down_proj")]
    if cfg == 4:   # decode regime, Llama2-13B shapes
        return 3, [LayerShape(64, 5120, 5120, 28, 8, 2, 2.0, "bf16", "uniform", "attn_proj"),
                   LayerShape(64, 5120, 13824, 28, 8, 2, 2.0, "bf16", "uniform", "mlp_up")]
    if cfg == 5:   # full Llama3-8B block, r=16, mixed routing
        T, r = 16384, 16
        mk = lambda di, do, rt, nm: LayerShape(T, di, do, 28, r, 2, 2.0, "bf16", rt, nm)
        return 4, [mk(4096, 4096, "uniform", "q_proj"), mk(4096, 1024, "uniform", "k_proj"),
                   mk(4096, 1024, "uniform", "v_proj"), mk(4096, 4096, "uniform", "o_proj"),
                   mk(4096, 14336, "zipf", "gate_proj"), mk(4096, 14336, "zipf", "up_proj"),
                   mk(14336, 4096, "zipf", "down_proj")]
    raise ValueError(f"unknown config {cfg}")
