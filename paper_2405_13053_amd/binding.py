"""ctypes binding of libmeteora.so: same names as the C ABI, argument marshalling only.

PyTorch is used for device memory and the current stream; every step of the
layer runs inside the library's HIP kernels.  There is no fallback: if the
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmeteora.so")
_lib = None

F32, BF16 = 0, 1


class MeteoraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = load_library().meteora_status_string(status).decode()
        super().__init__(f"{where}: {msg} (status {status})")


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libmeteora.so built in-tree; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} not found: build it first (python -m paper_2405_13053_amd.build "
            "or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(_LIB_PATH)
    c = ctypes
    vp, i, f, sz = c.c_void_p, c.c_int, c.c_float, c.c_size_t
    lib.meteora_version.restype = i
    lib.meteora_status_string.restype = c.c_char_p
    lib.meteora_status_string.argtypes = [i]
    lib.meteora_workspace_bytes.restype = sz
    lib.meteora_workspace_bytes.argtypes = [i, i, i, i, i, i, i]
    lib.meteora_gate_topk.restype = i
    lib.meteora_gate_topk.argtypes = [vp, vp, vp, i, i, i, i, i, f, vp, vp, vp, vp, sz, vp]
    lib.meteora_bucket_tokens.restype = i
    lib.meteora_bucket_tokens.argtypes = [vp, i, i, i, vp, vp, vp, vp, vp, sz, vp]
    lib.meteora_bucket_tokens_noalloc.restype = i
    lib.meteora_bucket_tokens_noalloc.argtypes = [vp, i, i, i, vp, vp, vp, vp, vp]
    lib.meteora_lora_forward.restype = i
    lib.meteora_lora_forward.argtypes = [vp, vp, vp, vp, vp, i, i, i, i, i, i, f, i, vp, i, vp, sz, vp]
    lib.meteora_linear_forward.restype = i
    lib.meteora_linear_forward.argtypes = [vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, f, f, i, vp, vp, vp, vp, sz, vp]
    lib.meteora_init.restype = i
    lib.meteora_init.argtypes = [i]
    lib.meteora_workspace_regions.restype = i
    lib.meteora_workspace_regions.argtypes = [i, i, i, i, i, i, i, i, vp, vp, vp, vp, i]
    lib.meteora_packed_bytes.restype = sz
    lib.meteora_packed_bytes.argtypes = [i, i, i, i, i]
    lib.meteora_pack_weights.restype = i
    lib.meteora_pack_weights.argtypes = [vp, vp, vp, i, i, i, i, i, vp, sz, vp]
    lib.meteora_linear_forward_packed.restype = i
    lib.meteora_linear_forward_packed.argtypes = [vp, vp, vp, vp, vp, vp, vp, sz, i, i, i, i, i, i, f, f, i, vp, vp,
                                                  vp, vp, sz, vp]
    lib.meteora_group_workspace_bytes.restype = sz
    lib.meteora_group_workspace_bytes.argtypes = [vp, i, i, i, i, i, i, i]
    lib.meteora_linear_forward_group.restype = i
    lib.meteora_linear_forward_group.argtypes = [vp, vp, i, i, i, i, i, i, f, f, i, vp, sz, vp]
    lib.meteora_gate_backward_workspace_bytes.restype = sz
    lib.meteora_gate_backward_workspace_bytes.argtypes = [i, i, i, i, i, i, i]
    lib.meteora_gate_backward.restype = i
    lib.meteora_gate_backward.argtypes = [vp, vp, vp, vp, vp, sz, vp, vp, vp, f, i, i, i, i, i, i, f, i, vp, vp, vp,
                                          vp, vp, vp, vp, vp, sz, vp, sz, vp]
    lib.meteora_variant_workspace_bytes.restype = sz
    lib.meteora_variant_workspace_bytes.argtypes = [i, i, i, i, i, i, i, i]
    lib.meteora_variant_forward.restype = i
    lib.meteora_variant_forward.argtypes = [i, vp, vp, vp, vp, vp, vp, i, i, i, i, i, i, f, i, vp, vp, vp, vp, sz, vp]
    lib.meteora_base_gemm.restype = i
    lib.meteora_base_gemm.argtypes = [vp, vp, i, i, i, i, vp, vp]
    lib.meteora_stage_count.restype = i
    lib.meteora_stage_name.restype = c.c_char_p
    lib.meteora_stage_name.argtypes = [i]
    lib.meteora_stage_timing_enable.restype = i
    lib.meteora_stage_timing_enable.argtypes = [i]
    lib.meteora_stage_timing_read.restype = i
    lib.meteora_stage_timing_read.argtypes = [vp, vp, vp]
    _lib = lib
    return lib


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _p(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _chk(t: Optional[torch.Tensor], name: str, dtype=None, shape=None):
    if t is None:
        return
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def workspace_bytes(T, d_in, d_out, N, r, k, dtype) -> int:
    dt = BF16 if dtype in (torch.bfloat16, BF16, "bf16") else F32
    return int(load_library().meteora_workspace_bytes(T, d_in, d_out, N, r, k, dt))


def init(device: int = -1) -> None:
    """meteora_init: per-device set-up ahead of the first launch (needed before a first call is graph-captured)."""
    st = load_library().meteora_init(int(device))
    if st != 0:
        raise MeteoraError(st, "meteora_init")


def workspace_regions(T, d_in, d_out, N, r, k, dtype, with_packed: bool = False):
    """meteora_workspace_regions: list of (name, offset, reserved, written) or None for unsupported arguments."""
    dt = BF16 if dtype in (torch.bfloat16, BF16, "bf16") else F32
    cap = 64
    names = (ctypes.c_char_p * cap)()
    off = (ctypes.c_size_t * cap)()
    res = (ctypes.c_size_t * cap)()
    wr = (ctypes.c_size_t * cap)()
    n = load_library().meteora_workspace_regions(T, d_in, d_out, N, r, k, dt, int(bool(with_packed)), names, off,
                                                 res, wr, cap)
    if n < 0:
        return None
    return [(names[j].decode(), int(off[j]), int(res[j]), int(wr[j])) for j in range(n)]


def _ws(ws: Optional[torch.Tensor], need: int, device) -> torch.Tensor:
    if ws is None:
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return ws


def gate_topk(x, W_gate, gate_bias, k: int, inv_temperature: float = 1.0, want_logits: bool = False,
              ws: Optional[torch.Tensor] = None):
    """meteora_gate_topk: returns (topk_idx[T,k] i32, topk_w[T,k] f32, logits[T,N] f32 or None)."""
    T, d_in = x.shape
    N = W_gate.shape[1]
    _chk(x, "x"); _chk(W_gate, "W_gate", torch.float32, (d_in, N)); _chk(gate_bias, "gate_bias", torch.float32, (N,))
    idx = torch.empty((T, k), dtype=torch.int32, device=x.device)
    w = torch.empty((T, k), dtype=torch.float32, device=x.device)
    logits = torch.empty((T, N), dtype=torch.float32, device=x.device) if want_logits else None
    ws = _ws(ws, workspace_bytes(T, d_in, 8, N, 1, k, x.dtype), x.device)
    st = load_library().meteora_gate_topk(_p(x), _p(W_gate), _p(gate_bias), T, d_in, N, k, _dt(x),
                                          float(inv_temperature), _p(idx), _p(w), _p(logits), _p(ws),
                                          ws.numel(), _stream())
    if st != 0:
        raise MeteoraError(st, "meteora_gate_topk")
    return idx, w, logits


def bucket_tokens(topk_idx, N: int, ws: Optional[torch.Tensor] = None):
    """meteora_bucket_tokens: returns (counts[N], offsets[N+1], bucket_tok[T*k], bucket_slot[T*k])."""
    _chk(topk_idx, "topk_idx", torch.int32)
    T, k = topk_idx.shape
    dev = topk_idx.device
    counts = torch.empty(N, dtype=torch.int32, device=dev)
    offsets = torch.empty(N + 1, dtype=torch.int32, device=dev)
    tok = torch.empty(T * k, dtype=torch.int32, device=dev)
    slot = torch.empty(T * k, dtype=torch.int32, device=dev)
    ws = _ws(ws, workspace_bytes(T, 8, 8, N, 1, k, torch.float32), dev)
    st = load_library().meteora_bucket_tokens(_p(topk_idx), T, k, N, _p(counts), _p(offsets), _p(tok), _p(slot),
                                              _p(ws), ws.numel(), _stream())
    if st != 0:
        raise MeteoraError(st, "meteora_bucket_tokens")
    return counts, offsets, tok, slot


def bucket_tokens_noalloc(topk_idx, N: int, out=None):
    """meteora_bucket_tokens_noalloc: as bucket_tokens, on the library's own fixed scratch.  `out` = the four
    result tensors (counts, offsets, bucket_tok, bucket_slot) if the caller has them already."""
    _chk(topk_idx, "topk_idx", torch.int32)
    T, k = topk_idx.shape
    dev = topk_idx.device
    if out is None:
        out = (torch.empty(N, dtype=torch.int32, device=dev), torch.empty(N + 1, dtype=torch.int32, device=dev),
               torch.empty(T * k, dtype=torch.int32, device=dev), torch.empty(T * k, dtype=torch.int32, device=dev))
    counts, offsets, tok, slot = out
    st = load_library().meteora_bucket_tokens_noalloc(_p(topk_idx), T, k, N, _p(counts), _p(offsets), _p(tok),
                                                      _p(slot), _stream())
    if st != 0:
        raise MeteoraError(st, "meteora_bucket_tokens_noalloc")
    return counts, offsets, tok, slot


def lora_forward(x, A, B, topk_idx, topk_w, scale: float, out: Optional[torch.Tensor] = None,
                 accumulate: bool = False, ws: Optional[torch.Tensor] = None):
    """meteora_lora_forward: out (+)= scale * sum_j w_j (x A_j) B_j for the given routing."""
    T, d_in = x.shape
    N, _, r = A.shape
    d_out = B.shape[2]
    k = topk_idx.shape[1]
    _chk(x, "x"); _chk(A, "A", x.dtype, (N, d_in, r)); _chk(B, "B", x.dtype, (N, r, d_out))
    _chk(topk_idx, "topk_idx", torch.int32, (T, k)); _chk(topk_w, "topk_w", torch.float32, (T, k))
    if out is None:
        if accumulate:
            raise ValueError("accumulate needs an existing out")
        out = torch.empty((T, d_out), dtype=x.dtype, device=x.device)
    _chk(out, "out", x.dtype, (T, d_out))
    ws = _ws(ws, workspace_bytes(T, d_in, d_out, N, r, k, x.dtype), x.device)
    st = load_library().meteora_lora_forward(_p(x), _p(A), _p(B), _p(topk_idx), _p(topk_w), T, d_in, d_out, N,
                                             r, k, float(scale), _dt(x), _p(out), int(bool(accumulate)), _p(ws),
                                             ws.numel(), _stream())
    if st != 0:
        raise MeteoraError(st, "meteora_lora_forward")
    return out


def packed_bytes(d_in, d_out, N, r, dtype) -> int:
    dt = BF16 if dtype in (torch.bfloat16, BF16, "bf16") else F32
    return int(load_library().meteora_packed_bytes(d_in, d_out, N, r, dt))


def pack_weights(W_gate, A, B, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """meteora_pack_weights: the kernel-side layouts of W_gate, A, B, built once per set of adapters."""
    N, d_in, r = A.shape
    d_out = B.shape[2]
    _chk(W_gate, "W_gate", torch.float32, (d_in, N)); _chk(A, "A"); _chk(B, "B", A.dtype, (N, r, d_out))
    nbytes = packed_bytes(d_in, d_out, N, r, A.dtype)
    if out is None:
        out = torch.empty((max(nbytes, 1),), dtype=torch.uint8, device=A.device)
    st = load_library().meteora_pack_weights(_p(W_gate), _p(A), _p(B), d_in, d_out, N, r, _dt(A), _p(out),
                                             out.numel(), _stream())
    if st != 0:
        raise MeteoraError(st, "meteora_pack_weights")
    return out


def linear_forward(x, W, W_gate, gate_bias, A, B, k: int, scale: float, out: Optional[torch.Tensor] = None,
                   ws: Optional[torch.Tensor] = None, return_routing: bool = False,
                   packed: Optional[torch.Tensor] = None, inv_temperature: float = 1.0):
    """meteora_linear_forward / meteora_linear_forward_packed (if `packed` is given): the whole layer (Eq. 2)."""
    T, d_in = x.shape
    d_out = W.shape[0]
    N, _, r = A.shape
    _chk(x, "x"); _chk(W, "W", x.dtype, (d_out, d_in)); _chk(W_gate, "W_gate", torch.float32, (d_in, N))
    _chk(gate_bias, "gate_bias", torch.float32, (N,))
    _chk(A, "A", x.dtype, (N, d_in, r)); _chk(B, "B", x.dtype, (N, r, d_out))
    _chk(packed, "packed", torch.uint8)
    if out is None:
        out = torch.empty((T, d_out), dtype=x.dtype, device=x.device)
    _chk(out, "out", x.dtype, (T, d_out))
    idx = w = None
    if return_routing:
        idx = torch.empty((T, k), dtype=torch.int32, device=x.device)
        w = torch.empty((T, k), dtype=torch.float32, device=x.device)
    ws = _ws(ws, workspace_bytes(T, d_in, d_out, N, r, k, x.dtype), x.device)
    lib = load_library()
    if packed is None:
        st = lib.meteora_linear_forward(_p(x), _p(W), _p(W_gate), _p(gate_bias), _p(A), _p(B), T, d_in, d_out, N, r,
                                        k, float(scale), float(inv_temperature), _dt(x), _p(out), _p(idx), _p(w),
                                        _p(ws), ws.numel(), _stream())
    else:
        st = lib.meteora_linear_forward_packed(_p(x), _p(W), _p(W_gate), _p(gate_bias), _p(A), _p(B), _p(packed),
                                               packed.numel(), T, d_in, d_out, N, r, k, float(scale),
                                               float(inv_temperature), _dt(x), _p(out), _p(idx), _p(w), _p(ws),
                                               ws.numel(), _stream())
    if st != 0:
        raise MeteoraError(st, "meteora_linear_forward")
    return (out, idx, w) if return_routing else out


class GroupMember(ctypes.Structure):
    """meteora_group_member of include/meteora.h."""
    _fields_ = [("W", ctypes.c_void_p), ("W_gate", ctypes.c_void_p), ("gate_bias", ctypes.c_void_p),
                ("A", ctypes.c_void_p), ("B", ctypes.c_void_p), ("packed", ctypes.c_void_p),
                ("packed_bytes", ctypes.c_size_t), ("d_out", ctypes.c_int), ("out", ctypes.c_void_p),
                ("topk_idx_out", ctypes.c_void_p), ("topk_w_out", ctypes.c_void_p)]


def group_workspace_bytes(d_outs: Sequence[int], T: int, d_in: int, N: int, r: int, k: int, dtype) -> int:
    """meteora_group_workspace_bytes."""
    arr = (ctypes.c_int * len(d_outs))(*d_outs)
    dt = BF16 if dtype in (torch.bfloat16, BF16, "bf16") else F32
    return int(load_library().meteora_group_workspace_bytes(arr, len(d_outs), T, d_in, N, r, k, dt))


def linear_forward_group(x, members, k: int, scale: float, ws: Optional[torch.Tensor] = None,
                         return_routing: bool = False, inv_temperature: float = 1.0):
    """meteora_linear_forward_group: layers that share x.  `members` is a sequence of dicts with W, W_gate,
    gate_bias (or None), A, B, packed (or None) and optionally out; returns the list of outputs
    (or of (out, idx, w) with return_routing)."""
    T, d_in = x.shape
    N, _, r = members[0]["A"].shape
    _chk(x, "x")
    arr = (GroupMember * len(members))()
    keep, res = [], []
    for g, mb in enumerate(members):
        W, Wg, bias, A, B, packed = mb["W"], mb["W_gate"], mb.get("gate_bias"), mb["A"], mb["B"], mb.get("packed")
        d_out = W.shape[0]
        _chk(W, "W", x.dtype, (d_out, d_in)); _chk(Wg, "W_gate", torch.float32, (d_in, N))
        _chk(bias, "gate_bias", torch.float32, (N,))
        _chk(A, "A", x.dtype, (N, d_in, r)); _chk(B, "B", x.dtype, (N, r, d_out)); _chk(packed, "packed", torch.uint8)
        out = mb.get("out")
        if out is None:
            out = torch.empty((T, d_out), dtype=x.dtype, device=x.device)
        _chk(out, "out", x.dtype, (T, d_out))
        idx = w = None
        if return_routing:
            idx = torch.empty((T, k), dtype=torch.int32, device=x.device)
            w = torch.empty((T, k), dtype=torch.float32, device=x.device)
        ptr = lambda t: None if t is None else t.data_ptr()
        arr[g] = GroupMember(ptr(W), ptr(Wg), ptr(bias), ptr(A), ptr(B), ptr(packed),
                             packed.numel() if packed is not None else 0, d_out, ptr(out), ptr(idx), ptr(w))
        keep.append((out, idx, w))
        res.append((out, idx, w) if return_routing else out)
    ws = _ws(ws, group_workspace_bytes([mb["W"].shape[0] for mb in members], T, d_in, N, r, k, x.dtype), x.device)
    st = load_library().meteora_linear_forward_group(_p(x), arr, len(members), T, d_in, N, r, k, float(scale),
                                                     float(inv_temperature), _dt(x), _p(ws), ws.numel(), _stream())
    if st != 0:
        raise MeteoraError(st, "meteora_linear_forward_group")
    return res


def gate_backward_workspace_bytes(T, d_in, d_out, N, r, k, dtype) -> int:
    dt = BF16 if dtype in (torch.bfloat16, BF16, "bf16") else F32
    return int(load_library().meteora_gate_backward_workspace_bytes(T, d_in, d_out, N, r, k, dt))


def gate_backward(x, dy, gate_bias, B, packed, k: int, scale: float, labels=None, beta: float = 0.0,
                  topk_idx=None, topk_w=None, want_dbias: bool = True, want_d_logits: bool = False,
                  ws: Optional[torch.Tensor] = None, forward_ws: Optional[torch.Tensor] = None,
                  A=None, W_gate=None, W_t=None, want_dx: bool = False):
    """meteora_gate_backward: (dW_gate[d_in,N], dbias[N] or None, d_logits[T,N] or None), all fp32; with
    want_dx (needs A, W_gate and W_t = W transposed, [d_in,d_out]) a fourth entry dx[T,d_in] in x's dtype."""
    T, d_in = x.shape
    N, r, d_out = B.shape
    _chk(x, "x"); _chk(dy, "dy", x.dtype, (T, d_out)); _chk(gate_bias, "gate_bias", torch.float32, (N,))
    _chk(B, "B", x.dtype, (N, r, d_out)); _chk(packed, "packed", torch.uint8)
    _chk(labels, "labels", torch.int32, (T,))
    _chk(topk_idx, "topk_idx", torch.int32, (T, k)); _chk(topk_w, "topk_w", torch.float32, (T, k))
    _chk(forward_ws, "forward_ws", torch.uint8)
    dxo = None
    if want_dx:
        _chk(A, "A", x.dtype, (N, d_in, r)); _chk(W_gate, "W_gate", torch.float32, (d_in, N))
        _chk(W_t, "W_t", x.dtype, (d_in, d_out))
        if A is None or W_gate is None or W_t is None:
            raise ValueError("want_dx needs A, W_gate and W_t")
        dxo = torch.empty((T, d_in), dtype=x.dtype, device=x.device)
    need = gate_backward_workspace_bytes(T, d_in, d_out, N, r, k, x.dtype)
    if need == 0 and T > 0:
        raise MeteoraError(2, "meteora_gate_backward_workspace_bytes")
    ws = _ws(ws, need, x.device)
    dW = torch.empty((d_in, N), dtype=torch.float32, device=x.device)
    db = torch.empty((N,), dtype=torch.float32, device=x.device) if want_dbias else None
    dl = torch.empty((T, N), dtype=torch.float32, device=x.device) if want_d_logits else None
    st = load_library().meteora_gate_backward(_p(x), _p(dy), _p(gate_bias), _p(B), _p(packed),
                                              0 if packed is None else packed.numel(), _p(topk_idx), _p(topk_w),
                                              _p(labels), float(beta), T, d_in, d_out, N, r, k, float(scale),
                                              _dt(x), _p(dW), _p(db), _p(dl), _p(A if want_dx else None),
                                              _p(W_gate if want_dx else None), _p(W_t if want_dx else None),
                                              _p(dxo), _p(forward_ws),
                                              0 if forward_ws is None else forward_ws.numel(), _p(ws), ws.numel(),
                                              _stream())
    if st != 0:
        raise MeteoraError(st, "meteora_gate_backward")
    return (dW, db, dl, dxo) if want_dx else (dW, db, dl)


LOOP_ORIGINAL, BMM_GATHER = 0, 1


def variant_workspace_bytes(variant: int, T, d_in, d_out, N, r, k, dtype) -> int:
    dt = BF16 if dtype in (torch.bfloat16, BF16, "bf16") else F32
    return int(load_library().meteora_variant_workspace_bytes(int(variant), T, d_in, d_out, N, r, k, dt))


def variant_forward(variant: int, x, W, W_gate, gate_bias, A, B, k: int, scale: float,
                    out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None,
                    return_routing: bool = False):
    """meteora_variant_forward: the layer through one of the paper's own schedules (LOOP_ORIGINAL, BMM_GATHER)."""
    T, d_in = x.shape
    d_out = W.shape[0]
    N, _, r = A.shape
    _chk(x, "x"); _chk(W, "W", x.dtype, (d_out, d_in)); _chk(W_gate, "W_gate", torch.float32, (d_in, N))
    _chk(gate_bias, "gate_bias", torch.float32, (N,))
    _chk(A, "A", x.dtype, (N, d_in, r)); _chk(B, "B", x.dtype, (N, r, d_out))
    if out is None:
        out = torch.empty((T, d_out), dtype=x.dtype, device=x.device)
    _chk(out, "out", x.dtype, (T, d_out))
    idx = w = None
    if return_routing:
        idx = torch.empty((T, k), dtype=torch.int32, device=x.device)
        w = torch.empty((T, k), dtype=torch.float32, device=x.device)
    need = variant_workspace_bytes(variant, T, d_in, d_out, N, r, k, x.dtype)
    if need == 0 and T > 0:
        raise MeteoraError(2, "meteora_variant_workspace_bytes")
    ws = _ws(ws, need, x.device)
    st = load_library().meteora_variant_forward(int(variant), _p(x), _p(W), _p(W_gate), _p(gate_bias), _p(A), _p(B),
                                                T, d_in, d_out, N, r, k, float(scale), _dt(x), _p(out), _p(idx),
                                                _p(w), _p(ws), ws.numel(), _stream())
    if st != 0:
        raise MeteoraError(st, "meteora_variant_forward")
    return (out, idx, w) if return_routing else out


def base_gemm(x, W, out: Optional[torch.Tensor] = None):
    """meteora_base_gemm: out = x W^T (W stored [d_out, d_in])."""
    T, d_in = x.shape
    d_out = W.shape[0]
    _chk(x, "x"); _chk(W, "W", x.dtype, (d_out, d_in))
    if out is None:
        out = torch.empty((T, d_out), dtype=x.dtype, device=x.device)
    _chk(out, "out", x.dtype, (T, d_out))
    st = load_library().meteora_base_gemm(_p(x), _p(W), T, d_in, d_out, _dt(x), _p(out), _stream())
    if st != 0:
        raise MeteoraError(st, "meteora_base_gemm")
    return out


def stage_timing_enable(on: bool) -> None:
    """meteora_stage_timing_enable: record hipEvents around each stage of the next calls."""
    st = load_library().meteora_stage_timing_enable(int(bool(on)))
    if st != 0:
        raise MeteoraError(st, "meteora_stage_timing_enable")


def stage_timing_read():
    """meteora_stage_timing_read: {stage: (ms_sum, launches)}, calls."""
    lib = load_library()
    n = lib.meteora_stage_count()
    ms = (ctypes.c_float * n)()
    launches = (ctypes.c_int * n)()
    calls = ctypes.c_int(0)
    st = lib.meteora_stage_timing_read(ms, launches, ctypes.byref(calls))
    if st != 0:
        raise MeteoraError(st, "meteora_stage_timing_read")
    return {lib.meteora_stage_name(s).decode(): (float(ms[s]), int(launches[s])) for s in range(n)}, calls.value
