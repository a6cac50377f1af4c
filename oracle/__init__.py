"""ctypes front end of the CPU oracle (oracle/meteora_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and
by bench.py's cpu_baseline leg.  The GPU library and its Python binding never
import this package.

All array arguments are numpy arrays.  x, W, A, B, W_gate, bias are float32
arrays holding exactly the values the storage dtype holds (a bf16 tensor is
passed as the fp32 array of its values); all results are double unless noted.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "meteora_oracle.c")
_LIB = os.path.join(_HERE, "libmeteora_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over tokens only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared",
                               "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _rows(rows, T):
    if rows is None:
        return None, T
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    if rows.size and (rows.min() < 0 or rows.max() >= T):
        raise ValueError("row index out of range")
    return rows, int(rows.size)


def gate_logits(x, W_gate, bias=None, rows=None) -> np.ndarray:
    """G(x) = x*W_gate (+bias) in double, [nrows, N]  (Sec. 3.1)."""
    x, W_gate = _f32(x), _f32(W_gate)
    T, d_in = x.shape
    assert W_gate.shape[0] == d_in
    N = W_gate.shape[1]
    bias = None if bias is None else _f32(bias)
    rows, n = _rows(rows, T)
    out = np.empty((n, N), dtype=np.float64)
    _load().oracle_gate_logits(_ptr(x), _ptr(W_gate), _ptr(bias), ctypes.c_int(d_in),
                               ctypes.c_int(N), _ptr(rows), ctypes.c_int(n), _ptr(out))
    return out


def topk_softmax(logits32, k: int, temperature: float = 1.0):
    """Top-k indices (descending logit, ties -> lower index) and Eq. 3 weights."""
    g = _f32(logits32)
    n, N = g.shape
    if not (1 <= k <= N):
        raise ValueError("need 1 <= k <= N")
    idx = np.empty((n, k), dtype=np.int32)
    w = np.empty((n, k), dtype=np.float64)
    _load().oracle_topk_softmax(_ptr(g), ctypes.c_int(n), ctypes.c_int(N), ctypes.c_int(k),
                                ctypes.c_double(1.0 / temperature), _ptr(idx), _ptr(w))
    return idx, w


def bucket(idx, N: int):
    """Stable per-adapter (token, slot) lists: counts, offsets, bucket_tok, bucket_slot."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    T, k = idx.shape
    if idx.size and (idx.min() < 0 or idx.max() >= N):
        raise ValueError("adapter index out of range")
    counts = np.empty(N, dtype=np.int32)
    offsets = np.empty(N + 1, dtype=np.int32)
    tok = np.empty(T * k, dtype=np.int32)
    slot = np.empty(T * k, dtype=np.int32)
    _load().oracle_bucket(_ptr(idx), ctypes.c_int(T), ctypes.c_int(k), ctypes.c_int(N),
                          _ptr(counts), _ptr(offsets), _ptr(tok), _ptr(slot))
    return counts, offsets, tok, slot


def base(x, W, rows=None) -> np.ndarray:
    """o_base = x*W_base with W stored [d_out, d_in]; double, [nrows, d_out]."""
    x, W = _f32(x), _f32(W)
    T, d_in = x.shape
    d_out = W.shape[0]
    assert W.shape[1] == d_in
    rows, n = _rows(rows, T)
    y = np.empty((n, d_out), dtype=np.float64)
    _load().oracle_base(_ptr(x), _ptr(W), ctypes.c_int(d_in), ctypes.c_int(d_out),
                        _ptr(rows), ctypes.c_int(n), _ptr(y))
    return y


def lora_delta(x, A, B, idx, w, scale: float, rows=None, return_h: bool = False):
    """s * sum_slot w * ((x*A_a)*B_a) for the evaluated rows (idx, w given per evaluated row)."""
    x, A, B = _f32(x), _f32(A), _f32(B)
    T, d_in = x.shape
    N, d_in2, r = A.shape
    N2, r2, d_out = B.shape
    assert d_in2 == d_in and N2 == N and r2 == r
    rows, n = _rows(rows, T)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    w = np.ascontiguousarray(w, dtype=np.float64)
    k = idx.shape[1]
    assert idx.shape == (n, k) and w.shape == (n, k)
    if idx.size and (idx.min() < 0 or idx.max() >= N):
        raise ValueError("adapter index out of range")
    delta = np.empty((n, d_out), dtype=np.float64)
    h = np.empty((n, k, r), dtype=np.float64) if return_h else None
    _load().oracle_lora_delta(_ptr(x), _ptr(A), _ptr(B), _ptr(idx), _ptr(w), ctypes.c_int(d_in),
                              ctypes.c_int(d_out), ctypes.c_int(r), ctypes.c_int(k),
                              ctypes.c_double(scale), _ptr(rows), ctypes.c_int(n), _ptr(delta),
                              _ptr(h))
    return (delta, h) if return_h else delta


def linear_forward(x, W, W_gate, bias, A, B, k: int, scale: float, rows=None, temperature: float = 1.0):
    """Whole layer (Eq. 2) on the given rows.

    temperature: the softmax temperature of App. A.6 (1.0 = Eq. 3 as printed).
    Returns dict(y[nrows,d_out] f64, logits[nrows,N] f32, idx[nrows,k] i32, w[nrows,k] f64).
    """
    x, W, W_gate, A, B = _f32(x), _f32(W), _f32(W_gate), _f32(A), _f32(B)
    bias = None if bias is None else _f32(bias)
    T, d_in = x.shape
    d_out = W.shape[0]
    N, _, r = A.shape
    assert W.shape == (d_out, d_in) and W_gate.shape == (d_in, N)
    assert A.shape == (N, d_in, r) and B.shape == (N, r, d_out)
    if not (1 <= k <= N):
        raise ValueError("need 1 <= k <= N")
    rows, n = _rows(rows, T)
    y = np.empty((n, d_out), dtype=np.float64)
    logits = np.empty((n, N), dtype=np.float32)
    idx = np.empty((n, k), dtype=np.int32)
    w = np.empty((n, k), dtype=np.float64)
    s64 = np.empty((n, N), dtype=np.float64)
    delta = np.empty((n, d_out), dtype=np.float64)
    _load().oracle_linear_forward(_ptr(x), _ptr(W), _ptr(W_gate), _ptr(bias), _ptr(A), _ptr(B),
                                  ctypes.c_int(d_in), ctypes.c_int(d_out), ctypes.c_int(N),
                                  ctypes.c_int(r), ctypes.c_int(k), ctypes.c_double(scale),
                                  ctypes.c_double(1.0 / temperature),
                                  _ptr(rows), ctypes.c_int(n), _ptr(y), _ptr(logits), _ptr(idx),
                                  _ptr(w), _ptr(s64), _ptr(delta))
    return {"y": y, "logits": logits, "idx": idx, "w": w}
