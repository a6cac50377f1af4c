"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, sizes workspaces, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

import paper_2405_13053_amd as m

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, INVALID, UNSUPPORTED, WORKSPACE, HIP = range(5)
F32, BF16 = 0, 1


@pytest.fixture(scope="module")
def lib():
    return m.load_library()


def test_every_declared_symbol_is_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "meteora.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = sorted(set(re.findall(r"\b(meteora_[a-z_0-9]+)\s*\(", hdr)))
    assert {"meteora_gate_topk", "meteora_bucket_tokens", "meteora_lora_forward", "meteora_linear_forward",
            "meteora_base_gemm", "meteora_workspace_bytes", "meteora_packed_bytes", "meteora_pack_weights",
            "meteora_linear_forward_packed", "meteora_linear_forward_group",
            "meteora_group_workspace_bytes"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in meteora.h but not exported"


def test_version_and_status_strings(lib):
    assert lib.meteora_version() >= 100
    texts = {lib.meteora_status_string(s) for s in range(5)}
    assert len(texts) == 5


def test_workspace_bytes(lib):
    w = m.workspace_bytes(4096, 4096, 4096, 28, 8, 2, "bf16")
    assert w > 0 and w % 256 == 0
    assert m.workspace_bytes(8192, 4096, 4096, 28, 8, 2, "bf16") > w
    assert m.workspace_bytes(0, 4096, 4096, 28, 8, 2, "bf16") > 0            # T = 0 is legal
    assert m.workspace_bytes(64, 256, 256, 4, 8, 5, "f32") == 0              # k > N
    assert m.workspace_bytes(64, 250, 256, 4, 8, 2, "f32") == 0              # d_in % 8
    assert m.workspace_bytes(64, 256, 256, 65, 8, 2, "f32") == 0             # N > 64
    assert lib.meteora_workspace_bytes(64, 256, 256, 4, 8, 2, 7) == 0        # unknown dtype


def test_workspace_regions_hold_what_the_launches_write():
    """Walk batch sizes and layer shapes across every launch sequence (decode, split-K mid batches, dense routing,
    bucketed): each region of the workspace is at least as large as what the selected launches write into it
    (tile and K-split counts taken from the launch decisions), regions do not overlap, and all of them lie inside
    meteora_workspace_bytes."""
    Ts = [1, 7, 33, 64, 65, 100, 128, 129, 160, 200, 256, 257, 300, 400, 512, 513, 640, 700, 704, 768, 769, 1000,
          1024, 1150, 1151, 1500, 2000, 2048, 3000, 4096, 4097, 5000, 8192, 8193, 12000, 16384, 20000, 32768, 70000]
    dims = [(4096, 4096), (4096, 8), (4096, 256), (4096, 512), (4096, 1024), (4096, 14336), (14336, 4096),
            (5120, 5120), (5120, 13824), (512, 264), (1088, 520), (64, 72), (256, 136)]
    checked = 0
    for dtype in ("bf16", "f32"):
        for (N, r, k) in [(28, 8, 2), (28, 16, 2), (7, 32, 3), (64, 8, 8), (5, 5, 1)]:
            for d_in, d_out in dims:
                for T in Ts:
                    for with_packed in (False, True):
                        regs = m.workspace_regions(T, d_in, d_out, N, r, k, dtype, with_packed)
                        assert regs is not None
                        total = m.workspace_bytes(T, d_in, d_out, N, r, k, dtype)
                        end_prev = 0
                        for name, off, reserved, written in regs:
                            where = f"{name} T={T} {d_in}->{d_out} N={N} r={r} k={k} {dtype} packed={with_packed}"
                            assert off >= end_prev and off % 256 == 0, where
                            assert written <= reserved, f"{where}: writes {written} B into {reserved} B"
                            assert off + reserved <= total, where
                            end_prev = off + reserved
                        checked += 1
    assert checked > 5000
    # shapes whose split projection has more K splits than the routing products alone (d_out of one or two tiles)
    for T, d_in, d_out in ((3000, 4096, 256), (4096, 4096, 8)):
        regs = {n: (o, rsv, w) for n, o, rsv, w in m.workspace_regions(T, d_in, d_out, 28, 8, 2, "bf16", True)}
        assert regs["dpart"][2] <= regs["dpart"][1]


def test_init_without_a_device_reports_an_error(lib):
    """meteora_init is host code around HIP calls: on a machine with no GPU it returns an error code, it does not
    abort; with a GPU it succeeds and may be repeated."""
    import torch
    st = lib.meteora_init(-1)
    if torch.cuda.is_available():
        assert st == OK and lib.meteora_init(0) == OK
    else:
        assert st == HIP


# Fake, suitably aligned, never-dereferenced addresses: validation must reject before any launch.
P = ctypes.c_void_p(0x10000)
ODD = ctypes.c_void_p(0x10004)
WS = ctypes.c_void_p(0x100000)
BIG = 1 << 30


def gate(lib, x=P, Wg=P, bias=None, T=64, d=256, N=4, k=2, dt=F32, it=1.0, idx=P, w=P, lg=None, ws=WS, wsb=BIG):
    return lib.meteora_gate_topk(x, Wg, bias, T, d, N, k, dt, it, idx, w, lg, ws, wsb, None)


def test_gate_topk_validation(lib):
    assert gate(lib, x=None) == INVALID
    assert gate(lib, idx=None) == INVALID
    assert gate(lib, k=0) == INVALID
    assert gate(lib, k=5) == INVALID            # k > N
    assert gate(lib, T=-1) == INVALID
    assert gate(lib, it=float("nan")) == INVALID
    assert gate(lib, dt=3) == UNSUPPORTED
    assert gate(lib, d=250) == UNSUPPORTED
    assert gate(lib, N=65, k=2) == UNSUPPORTED
    assert gate(lib, N=16, k=9) == UNSUPPORTED
    assert gate(lib, x=ODD) == UNSUPPORTED
    assert gate(lib, ws=None) == WORKSPACE
    assert gate(lib, wsb=16) == WORKSPACE
    assert gate(lib, T=0) == OK                 # empty batch: nothing enqueued


def test_bucket_validation(lib):
    f = lambda idx=P, T=64, k=2, N=4, c=P, o=P, bt=P, bs=P, ws=WS, wsb=BIG: \
        lib.meteora_bucket_tokens(idx, T, k, N, c, o, bt, bs, ws, wsb, None)
    assert f(idx=None) == INVALID
    assert f(c=None) == INVALID
    assert f(k=5) == INVALID
    assert f(N=100, k=2) == UNSUPPORTED
    assert f(ws=None) == WORKSPACE
    assert f(wsb=0) == WORKSPACE
    assert f(T=0) == OK


def test_lora_and_linear_validation(lib):
    def lora(x=P, A=P, B=P, idx=P, w=P, T=64, di=256, do=256, N=4, r=8, k=2, s=2.0, dt=F32, out=P, acc=0,
             ws=WS, wsb=BIG):
        return lib.meteora_lora_forward(x, A, B, idx, w, T, di, do, N, r, k, s, dt, out, acc, ws, wsb, None)

    def lin(x=P, W=P, Wg=P, bias=None, A=P, B=P, T=64, di=256, do=256, N=4, r=8, k=2, s=2.0, dt=BF16, out=P,
            io=None, wo=None, ws=WS, wsb=BIG, it=1.0):
        return lib.meteora_linear_forward(x, W, Wg, bias, A, B, T, di, do, N, r, k, s, it, dt, out, io, wo, ws, wsb,
                                          None)

    for f in (lora, lin):
        assert f(x=None) == INVALID
        assert f(out=None) == INVALID
        assert f(k=0) == INVALID
        assert f(k=5) == INVALID
        assert f(r=0) == INVALID
        assert f(s=float("inf")) == INVALID
        assert f(do=100) == UNSUPPORTED
        assert f(r=65) == UNSUPPORTED
        assert f(dt=9) == UNSUPPORTED
        assert f(A=ODD) == UNSUPPORTED
        assert f(ws=None) == WORKSPACE
        assert f(wsb=1024) == WORKSPACE
        assert f(T=0) == OK
    assert lora(idx=None) == INVALID
    assert lora(acc=2) == INVALID
    assert lin(W=None) == INVALID
    assert lin(Wg=None) == INVALID
    assert lin(it=float("nan")) == INVALID and lin(it=float("inf")) == INVALID
    need = m.workspace_bytes(64, 256, 256, 4, 8, 2, "bf16")
    assert lin(wsb=need - 512) == WORKSPACE


def test_pack_weights_validation(lib):
    """Packed-weight entry points: sizes and argument checks (no launch happens on any error path)."""
    assert lib.meteora_packed_bytes(256, 256, 4, 8, F32) == 0          # fp32 reads the tensors as they are
    need = lib.meteora_packed_bytes(4096, 4096, 28, 8, BF16)
    # split gate weight (3 bf16 terms, 32 padded columns) + A in operand order (rank padded to 32) + B transposed
    assert need >= 4096 * 32 * 3 * 2 + 28 * 4096 * 32 * 2 + 4096 * 256 * 2
    assert lib.meteora_packed_bytes(4096, 4096, 65, 8, BF16) == 0      # unsupported shape
    assert m.packed_bytes(4096, 4096, 28, 8, "bf16") == need

    def pack(Wg=P, A=P, B=P, di=256, do=256, N=4, r=8, dt=BF16, pk=WS, pkb=BIG):
        return lib.meteora_pack_weights(Wg, A, B, di, do, N, r, dt, pk, pkb, None)

    assert pack(Wg=None) == INVALID and pack(A=None) == INVALID and pack(B=None) == INVALID
    assert pack(N=0) == INVALID
    assert pack(r=65) == UNSUPPORTED
    assert pack(dt=5) == UNSUPPORTED
    assert pack(A=ODD) == UNSUPPORTED
    assert pack(pk=None) == WORKSPACE
    assert pack(pkb=64) == WORKSPACE
    assert pack(dt=F32, pk=None, pkb=0) == OK                           # nothing to pack

    def linp(pk=WS, pkb=BIG, T=64, ws=WS, wsb=BIG, W=P):
        return lib.meteora_linear_forward_packed(P, W, P, None, P, P, pk, pkb, T, 256, 256, 4, 8, 2, 2.0, 1.0, BF16, P,
                                                 None, None, ws, wsb, None)

    assert linp(pkb=64) == WORKSPACE
    assert linp(pk=ODD) == WORKSPACE
    assert linp(W=None) == INVALID
    assert linp(wsb=1024) == WORKSPACE
    assert linp(T=0) == OK


def test_group_validation(lib):
    """Grouped entry point: sizes and argument checks on the host (no launch on any error path)."""
    from paper_2405_13053_amd.binding import GroupMember
    d_outs = (ctypes.c_int * 3)(4096, 1024, 1024)
    one = [lib.meteora_workspace_bytes(64, 4096, d, 28, 8, 2, BF16) for d in (4096, 1024, 1024)]
    need = lib.meteora_group_workspace_bytes(d_outs, 3, 64, 4096, 28, 8, 2, BF16)
    assert need >= max(one)                                # members may also run one after the other in it
    assert lib.meteora_group_workspace_bytes(d_outs, 0, 64, 4096, 28, 8, 2, BF16) == 0
    assert lib.meteora_group_workspace_bytes(None, 3, 64, 4096, 28, 8, 2, BF16) == 0
    assert lib.meteora_group_workspace_bytes(d_outs, 3, 64, 4096, 65, 8, 2, BF16) == 0   # unsupported member

    def member(W=P.value, Wg=P.value, A=P.value, B=P.value, pk=None, pkb=0, d_out=256, out=P.value):
        return GroupMember(W, Wg, None, A, B, pk, pkb, d_out, out, None, None)

    def call(ms, T=64, ws=WS, wsb=BIG, G=None, x=P, it=1.0):
        arr = (GroupMember * len(ms))(*ms)
        return lib.meteora_linear_forward_group(x, arr, len(ms) if G is None else G, T, 256, 4, 8, 2, 2.0, it, BF16,
                                                ws, wsb, None)

    two = [member(), member(d_out=264)]
    assert call(two, T=0) == OK
    assert call(two, G=0) == INVALID
    assert call(two, it=float("nan")) == INVALID
    assert call(two, x=None) == INVALID
    assert call([member(), member(W=None)]) == INVALID
    assert call([member(), member(out=None)]) == INVALID
    assert call([member(), member(d_out=7)]) == UNSUPPORTED
    assert call([member(), member(A=ODD.value)]) == UNSUPPORTED
    assert call([member(), member(pk=WS.value, pkb=64)]) == WORKSPACE
    assert call(two, wsb=1024) == WORKSPACE
    assert call(two, ws=None) == WORKSPACE
    assert lib.meteora_linear_forward_group(P, None, 2, 64, 256, 4, 8, 2, 2.0, 1.0, BF16, WS, BIG, None) == INVALID


def test_gate_backward_validation(lib):
    """Gate gradients: sizes and argument checks on the host (no launch on any error path)."""
    need = lib.meteora_gate_backward_workspace_bytes(4096, 4096, 4096, 28, 8, 2, BF16)
    assert need > 0
    # the two K-split partial arrays, the padded logit gradients and the slice partials of dW_gate all fit
    assert need >= 4096 * 320 * 4 + 4096 * 224 * 4 + 4096 * 32 * 4 + 4096 * 32 * 4
    assert lib.meteora_gate_backward_workspace_bytes(4096, 4096, 4096, 28, 8, 2, F32) == 0
    assert lib.meteora_gate_backward_workspace_bytes(4096, 4096, 4100, 28, 8, 2, BF16) == 0   # d_out % 64
    assert lib.meteora_gate_backward_workspace_bytes(4096, 4096, 4096, 28, 12, 2, BF16) == 0  # r % 8
    assert lib.meteora_gate_backward_workspace_bytes(4096, 4096, 4096, 40, 8, 2, BF16) == 0   # N > 32
    assert lib.meteora_gate_backward_workspace_bytes(70000, 4096, 4096, 28, 8, 2, BF16) == 0  # T > 65536
    pkb = lib.meteora_packed_bytes(256, 256, 4, 8, BF16)

    def call(x=P, dy=P, B=P, pk=WS, pkb=pkb, idx=None, w=None, T=64, d_out=256, N=4, r=8, k=2, scale=2.0, beta=0.0,
             dt=BF16, dW=P, ws=WS, wsb=BIG, fws=None, fwsb=0, A=None, Wg=None, Wt=None, dx=None):
        return lib.meteora_gate_backward(x, dy, None, B, pk, pkb, idx, w, None, beta, T, 256, d_out, N, r, k, scale, dt,
                                         dW, None, None, A, Wg, Wt, dx, fws, fwsb, ws, wsb, None)

    assert call(T=0) == OK
    assert call(x=None) == INVALID and call(dy=None) == INVALID and call(B=None) == INVALID
    assert call(pk=None) == INVALID and call(dW=None) == INVALID
    assert call(idx=P) == INVALID                          # routing: both arrays or neither
    assert call(k=5) == INVALID and call(scale=float("nan")) == INVALID and call(beta=float("inf")) == INVALID
    assert call(dt=F32) == UNSUPPORTED
    assert call(d_out=264) == UNSUPPORTED and call(r=4) == UNSUPPORTED and call(N=40, k=2) == UNSUPPORTED
    assert call(x=ODD) == UNSUPPORTED
    assert call(pkb=64) == WORKSPACE
    assert call(ws=None) == WORKSPACE and call(wsb=1024) == WORKSPACE
    assert call(T=128, fws=WS, fwsb=64) == WORKSPACE       # a forward workspace too small to hold the products
    assert call(T=0, fws=WS, fwsb=64) == OK
    assert call(dx=P) == INVALID and call(dx=P, A=P, Wg=P) == INVALID    # the input gradient needs A, W_gate and W_t
    assert call(dx=P, A=P, Wg=P, Wt=ODD) == UNSUPPORTED


def test_base_gemm_validation(lib):
    f = lambda x=P, W=P, T=64, di=256, do=256, dt=BF16, out=P: lib.meteora_base_gemm(x, W, T, di, do, dt, out, None)
    assert f(x=None) == INVALID and f(W=None) == INVALID and f(out=None) == INVALID
    assert f(T=-2) == INVALID
    assert f(di=12) == UNSUPPORTED
    assert f(dt=2) == UNSUPPORTED
    assert f(T=0) == OK


def test_bucket_tokens_noalloc_validation(lib):
    """The entry point on the library's own scratch rejects bad arguments and sizes beyond its fixed scratch on the
    host, before any HIP call."""
    f = lambda idx=P, T=64, k=2, N=4, c=P, o=P, bt=P, bs=P: lib.meteora_bucket_tokens_noalloc(idx, T, k, N, c, o, bt,
                                                                                          bs, None)
    assert f(idx=None) == INVALID and f(c=None) == INVALID and f(bs=None) == INVALID
    assert f(k=5) == INVALID and f(T=-1) == INVALID
    assert f(N=65, k=2) == UNSUPPORTED
    assert f(idx=ODD) == UNSUPPORTED
    assert f(T=65537) == 5 and f(T=1 << 20) == 5          # METEORA_ERR_TOO_LARGE
    assert b"fixed scratch" in lib.meteora_status_string(5)
    assert f(T=0) == OK


def test_variant_validation(lib):
    """The paper's schedules as baselines: sizes and argument checks on the host."""
    LOOP, BMM = 0, 1
    wl = lib.meteora_variant_workspace_bytes(LOOP, 4096, 4096, 4096, 28, 8, 2, BF16)
    wb = lib.meteora_variant_workspace_bytes(BMM, 4096, 4096, 4096, 28, 8, 2, BF16)
    assert wl > 0 and wb >= 4096 * 2 * 8 * (4096 + 4096) * 2        # the gathered copies of A and B
    assert lib.meteora_variant_workspace_bytes(2, 64, 256, 256, 4, 8, 2, BF16) == 0     # unknown variant
    assert lib.meteora_variant_workspace_bytes(LOOP, 64, 256, 256, 4, 5, 2, BF16) == 0  # r % 8

    def call(v=LOOP, x=P, W=P, A=P, T=64, r=8, k=2, s=2.0, ws=WS, wsb=BIG, out=P):
        return lib.meteora_variant_forward(v, x, W, P, None, A, P, T, 256, 256, 4, r, k, s, BF16, out, None, None, ws,
                                           wsb, None)

    for v in (LOOP, BMM):
        assert call(v, x=None) == INVALID and call(v, out=None) == INVALID and call(v, W=None) == INVALID
        assert call(v, k=5) == INVALID and call(v, s=float("nan")) == INVALID
        assert call(v, r=5) == UNSUPPORTED and call(v, A=ODD) == UNSUPPORTED
        assert call(v, ws=None) == WORKSPACE and call(v, wsb=1024) == WORKSPACE
        assert call(v, T=0) == OK
    assert call(v=7) == INVALID


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU: --gpus 2 exits with a message and a non-zero status, before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)
