"""Margin conditioning of test inputs (TEST INFRASTRUCTURE, part of the oracle side).

fp32 summation order differs between any two implementations of the gate, so
two logits closer than the summation noise can legitimately be ranked either
way.  To make "the top-k indices" a well-defined, order-independent quantity,
test inputs are conditioned: any token row whose oracle logits (double) have a
gap below ``delta`` between consecutive ranks 1..k+1 is re-drawn from the
seeded generator until no such row is left.  With logits ~N(0,1), N=28, k=2
and delta=1e-3 this touches about 1% of the rows and leaves the distribution
otherwise unchanged.  Exact ties (duplicated gate columns, zero gate) are
tested separately and are never conditioned.
"""
from __future__ import annotations

import numpy as np

from gen import inputs as _gen
from . import gate_logits


def small_margin_rows(logits64: np.ndarray, k: int, delta: float) -> np.ndarray:
    """Indices of rows whose ranks 1..k+1 contain two logits closer than delta."""
    N = logits64.shape[1]
    top = -np.sort(-logits64, axis=1)[:, :min(k + 1, N)]
    gaps = top[:, :-1] - top[:, 1:]
    return np.nonzero((gaps < delta).any(axis=1))[0].astype(np.int32)


def condition_margins(shape, seed: int, layer: int, x: np.ndarray, W_gate: np.ndarray,
                      bias=None, delta: float = 1e-3, max_attempts: int = 16) -> int:
    """Re-draw (in place) the rows of x with near-tied gate logits.  Returns #rows re-drawn."""
    bad = small_margin_rows(gate_logits(x, W_gate, bias), shape.k, delta)
    total = int(bad.size)
    attempt = 1
    while bad.size:
        if attempt > max_attempts:
            raise RuntimeError("margin conditioning did not converge")
        _gen.redraw_rows(x, bad, shape, seed, layer, attempt)
        sub = gate_logits(x, W_gate, bias, rows=bad)
        bad = bad[small_margin_rows(sub, shape.k, delta)]
        attempt += 1
    return total
