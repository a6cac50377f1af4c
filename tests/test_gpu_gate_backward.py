"""GPU parity of meteora_gate_backward (gate gradients of Sec. 3.2, Eq. 4) against oracle/gate_backward.py.

Both sides get the same bf16-exact inputs; the library computes in fp32 (fp32 accumulation of exact bf16
products, fp32 softmax), the oracle in float64, so the gradients agree to fp32 summation error:
max|g - g_ref| / max|g_ref| <= 1e-4 (sums of up to a few thousand terms of mixed sign).  The routing is
an integer decision: with margin-conditioned inputs it is the oracle's exactly.
"""
import numpy as np
import pytest
import torch

import paper_2405_13053_amd as m
from gen import inputs as gen
from oracle import gate_backward as oracle_bwd
from tests import util

LS = gen.LayerShape
pytestmark = pytest.mark.gpu

TOL = 1e-4

BACKWARD_SHAPES = [
    LS(1, 64, 64, 3, 8, 1, 2.0, "bf16", "uniform", "T=1-top1"),
    LS(37, 128, 192, 5, 8, 2, 2.0, "bf16", "uniform", "T=37-ragged-token-tile"),
    LS(129, 320, 256, 9, 24, 4, 0.7, "bf16", "zipf", "T=129-r24-k4-bias"),
    LS(700, 512, 256, 7, 32, 7, 1.0, "bf16", "uniform", "T=700-r32-k=N"),
    LS(1000, 1088, 576, 28, 8, 2, 2.0, "bf16", "zipf", "T=1000-ragged-K17"),
    LS(260, 384, 128, 28, 8, 8, 1.0, "bf16", "uniform", "T=260-k8"),
    LS(4500, 192, 320, 14, 16, 3, 2.0, "bf16", "zipf", "T=4500-r16-wide-tiles"),
    LS(300, 512, 256, 28, 16, 2, 2.0, "bf16", "uniform", "T=300-r16-N28-544-rows"),
]


def _rel(a: torch.Tensor, ref: np.ndarray) -> float:
    a = a.detach().to(torch.float64).cpu().numpy()
    return float(np.abs(a - ref).max() / max(np.abs(ref).max(), 1e-30))


def _case(shape, seed):
    ops, dev = util.make_case(shape, seed)
    dy, labels = gen.make_training_signals(shape, seed)
    dev["dy"] = util.to_dev(dy, torch.bfloat16)
    dev["labels"] = torch.from_numpy(labels).to("cuda")
    dev["packed"] = m.pack_weights(dev["W_gate"], dev["A"], dev["B"])
    return ops, dev, dy, labels


@pytest.mark.parametrize("shape", BACKWARD_SHAPES, ids=lambda s: s.name)
@pytest.mark.parametrize("beta", [0.0, 0.5])
def test_gate_backward_matches_oracle(shape, beta):
    ops, dev, dy, labels = _case(shape, seed=71)
    ref = oracle_bwd.gate_backward(ops["x"], dy, ops["W_gate"], ops["bias"], ops["A"], ops["B"], shape.k,
                                   shape.scale, labels, beta)
    dW, db, dl = m.gate_backward(dev["x"], dev["dy"], dev["bias"], dev["B"], dev["packed"], shape.k, shape.scale,
                                 labels=dev["labels"], beta=beta, want_d_logits=True)
    torch.cuda.synchronize()
    if shape.k == 1 and beta == 0.0:          # App. "Top-1 strategy": nothing reaches the gate
        assert not dW.any() and not db.any() and not dl.any()
        return
    assert _rel(dl, ref["d_logits"]) <= TOL
    assert _rel(dW, ref["dW_gate"]) <= TOL
    assert _rel(db, ref["dbias"]) <= TOL
    # each token's logit gradient sums to zero (both softmaxes are shift invariant)
    assert float(dl.sum(dim=1).abs().max()) <= 1e-5 * max(1.0, float(dl.abs().max()))


@pytest.mark.parametrize("shape", BACKWARD_SHAPES, ids=lambda s: s.name)
def test_gate_backward_input_gradient_matches_oracle(shape):
    """dx (bf16 storage, fp32 accumulation: the forward's output bar, 5e-3 of the largest entry) with a
    classification weight large enough that the gate term is a visible part of it; the other outputs are the
    same bits as without dx."""
    beta = 4.0
    ops, dev, dy, labels = _case(shape, seed=74)
    ref = oracle_bwd.gate_backward(ops["x"], dy, ops["W_gate"], ops["bias"], ops["A"], ops["B"], shape.k,
                                   shape.scale, labels, beta, W=ops["W"])
    W_t = dev["W"].t().contiguous()
    dW, db, dl, dx = m.gate_backward(dev["x"], dev["dy"], dev["bias"], dev["B"], dev["packed"], shape.k, shape.scale,
                                     labels=dev["labels"], beta=beta, want_d_logits=True, A=dev["A"],
                                     W_gate=dev["W_gate"], W_t=W_t, want_dx=True)
    dW2, db2, dl2 = m.gate_backward(dev["x"], dev["dy"], dev["bias"], dev["B"], dev["packed"], shape.k, shape.scale,
                                    labels=dev["labels"], beta=beta, want_d_logits=True)
    torch.cuda.synchronize()
    assert torch.equal(dW, dW2) and torch.equal(db, db2) and torch.equal(dl, dl2)
    assert _rel(dx, ref["dx"]) <= 5e-3
    # the three roads separately visible: without the gate and adapter parts the error would be far above the bar
    base_only = dy @ ops["W"].astype(np.float64)
    assert np.abs(ref["dx"] - base_only).max() / np.abs(ref["dx"]).max() > 2e-2


def test_gate_backward_input_gradient_gate_term_accuracy():
    """The gate term alone (dy = 0: no base and no adapter part, d_logits = beta * (softmax - onehot)) is computed
    from two-term bf16 splits, about 2^-16 of its size: what is left is the one bf16 rounding of dx, so nearly
    every entry IS the oracle's value rounded to bf16 (single-term bf16 operands, 2^-8, would miss most)."""
    shape = LS(200, 256, 192, 12, 8, 3, 2.0, "bf16", "zipf", "gate-term")
    ops, dev, dy, labels = _case(shape, seed=75)
    dy0 = np.zeros_like(dy)
    ref = oracle_bwd.gate_backward(ops["x"], dy0, ops["W_gate"], ops["bias"], ops["A"], ops["B"], shape.k,
                                   shape.scale, labels, 1.0, W=ops["W"])
    out = m.gate_backward(dev["x"], torch.zeros_like(dev["dy"]), dev["bias"], dev["B"], dev["packed"], shape.k,
                          shape.scale, labels=dev["labels"], beta=1.0, A=dev["A"], W_gate=dev["W_gate"],
                          W_t=dev["W"].t().contiguous(), want_dx=True)
    torch.cuda.synchronize()
    assert np.abs(ref["dx"]).max() > 0
    assert _rel(out[3], ref["dx"]) <= 5e-3
    rounded = gen.round_to_bf16(ref["dx"].astype(np.float32))
    got = out[3].to(torch.float32).cpu().numpy()
    assert np.mean(got != rounded) <= 0.02


def test_gate_backward_takes_the_forward_routing():
    """Given topk_idx / topk_w of the forward call the result equals the one from ranking again, and the routing
    the entry point would rank is the forward's (same logits, same routine)."""
    shape = LS(300, 256, 192, 12, 8, 3, 2.0, "bf16", "zipf", "given-routing")
    ops, dev, dy, labels = _case(shape, seed=72)
    _, idx, w = m.linear_forward(dev["x"], dev["W"], dev["W_gate"], dev["bias"], dev["A"], dev["B"], shape.k,
                                 shape.scale, return_routing=True, packed=dev["packed"])
    a = m.gate_backward(dev["x"], dev["dy"], dev["bias"], dev["B"], dev["packed"], shape.k, shape.scale,
                        labels=dev["labels"], beta=0.3, want_d_logits=True)
    b = m.gate_backward(dev["x"], dev["dy"], dev["bias"], dev["B"], dev["packed"], shape.k, shape.scale,
                        labels=dev["labels"], beta=0.3, topk_idx=idx, topk_w=w, want_d_logits=True)
    torch.cuda.synchronize()
    for u, v in zip(a, b):
        assert torch.equal(u, v)
    # a different routing changes the language-model part: the given one is really used
    idx2 = (idx + 1) % shape.N
    c = m.gate_backward(dev["x"], dev["dy"], dev["bias"], dev["B"], dev["packed"], shape.k, shape.scale,
                        topk_idx=idx2.contiguous(), topk_w=w, want_d_logits=True)
    d = m.gate_backward(dev["x"], dev["dy"], dev["bias"], dev["B"], dev["packed"], shape.k, shape.scale,
                        want_d_logits=True)
    assert not torch.equal(c[2], d[2])


@pytest.mark.parametrize("T,d_in,d_out,same_bits", [(300, 256, 192, True), (40, 256, 192, True), (300, 1024, 512, False)])
def test_gate_backward_reads_the_forward_products(T, d_in, d_out, same_bits):
    """With the forward call's workspace the products of x are not computed again.  T = 300, 256 -> 192: taken from
    the workspace, same bits as without it; T = 40: that forward path leaves none, the argument is ignored;
    T = 300, 1024 -> 512: the forward ran them inside its split-K projection launch with another number of K
    splits, so the sums differ in their last bits: equal to fp32 accuracy, and to the oracle as ever."""
    shape = LS(T, d_in, d_out, 12, 8, 3, 2.0, "bf16", "zipf", "forward-ws")
    ops, dev, dy, labels = _case(shape, seed=73)
    ws = torch.empty(m.workspace_bytes(T, shape.d_in, shape.d_out, shape.N, shape.r, shape.k, torch.bfloat16),
                     dtype=torch.uint8, device="cuda")
    _, idx, w = m.linear_forward(dev["x"], dev["W"], dev["W_gate"], dev["bias"], dev["A"], dev["B"], shape.k,
                                 shape.scale, return_routing=True, packed=dev["packed"], ws=ws)
    a = m.gate_backward(dev["x"], dev["dy"], dev["bias"], dev["B"], dev["packed"], shape.k, shape.scale,
                        labels=dev["labels"], beta=0.3, topk_idx=idx, topk_w=w, want_d_logits=True)
    b = m.gate_backward(dev["x"], dev["dy"], dev["bias"], dev["B"], dev["packed"], shape.k, shape.scale,
                        labels=dev["labels"], beta=0.3, topk_idx=idx, topk_w=w, want_d_logits=True, forward_ws=ws)
    torch.cuda.synchronize()
    for u, v in zip(a, b):
        if same_bits:
            assert torch.equal(u, v)
        else:
            assert float((u - v).abs().max()) <= 1e-5 * float(u.abs().max())
    if not same_bits:
        ref = oracle_bwd.gate_backward(ops["x"], dy, ops["W_gate"], ops["bias"], ops["A"], ops["B"], shape.k,
                                       shape.scale, labels, 0.3)
        assert _rel(b[0], ref["dW_gate"]) <= TOL and _rel(b[2], ref["d_logits"]) <= TOL
    if T > 64:   # and it is really read: a cleared workspace changes the result
        ws.zero_()
        c = m.gate_backward(dev["x"], dev["dy"], dev["bias"], dev["B"], dev["packed"], shape.k, shape.scale,
                            labels=dev["labels"], beta=0.3, topk_idx=idx, topk_w=w, want_d_logits=True, forward_ws=ws)
        assert not torch.equal(c[0], a[0])


def _sampled_check(shape, seed, cols):
    ops, dev, dy, labels = _case(shape, seed=seed)
    dW, db, dl = m.gate_backward(dev["x"], dev["dy"], dev["bias"], dev["B"], dev["packed"], shape.k, shape.scale,
                                 labels=dev["labels"], beta=0.25, want_d_logits=True)
    torch.cuda.synchronize()
    rows = np.linspace(0, shape.T - 1, 96).astype(np.int64)
    ref = oracle_bwd.gate_backward(ops["x"][rows], dy[rows], ops["W_gate"], ops["bias"], ops["A"], ops["B"], shape.k,
                                   shape.scale, labels[rows], 0.25)
    got = dl[torch.from_numpy(rows).to("cuda")]
    assert _rel(got, ref["d_logits"]) <= TOL
    dl64 = dl.to(torch.float64)
    assert _rel(db, dl64.sum(dim=0).cpu().numpy()) <= 1e-5
    cols = torch.tensor(cols, device="cuda")
    want = dev["x"][:, cols].to(torch.float64).T @ dl64
    assert _rel(dW[cols], want.cpu().numpy()) <= 1e-5


def test_gate_backward_full_size_sampled():
    """Config 2's layer (T = 4096, 4096 -> 4096, N = 28, r = 8, top-2): d_logits on sampled tokens against the
    oracle, dW_gate and dbias through properties that hold at any size: dbias = column sums of d_logits,
    sampled rows of dW_gate = x[:, c]^T d_logits in float64 from the library's own d_logits."""
    seed, shapes = gen.config_layers(2)
    _sampled_check(shapes[0], seed, [0, 1, 127, 128, 2049, 4095])


def test_gate_backward_many_tokens_sampled():
    """T = 40000 (wide product tiles, one K split, 313 token slices' worth of rows): index arithmetic at scale."""
    _sampled_check(LS(40000, 320, 192, 28, 8, 2, 2.0, "bf16", "zipf", "T=40000"), 77, [0, 63, 64, 129, 319])


def test_gate_backward_rejects_what_it_does_not_take():
    shape = LS(64, 128, 100, 5, 8, 2, 2.0, "bf16", "uniform", "d_out-not-64")
    assert m.gate_backward_workspace_bytes(shape.T, shape.d_in, shape.d_out, shape.N, shape.r, shape.k,
                                           torch.bfloat16) == 0
    assert m.gate_backward_workspace_bytes(64, 128, 128, 5, 8, 2, torch.float32) == 0
    assert m.gate_backward_workspace_bytes(64, 128, 128, 40, 8, 2, torch.bfloat16) == 0
    assert m.gate_backward_workspace_bytes(64, 128, 128, 5, 8, 2, torch.bfloat16) > 0


def test_training_step_replays_from_a_hip_graph():
    """Forward + gate gradients + dx captured once (no allocation by the library, no memset recorded) replay
    bit-identically on new x and dy, with eager work between the replays."""
    shape = LS(333, 512, 256, 12, 8, 2, 2.0, "bf16", "zipf", "graph-step")
    ops, dev, dy, labels = _case(shape, seed=76)
    bf = torch.bfloat16
    W_t = dev["W"].t().contiguous()
    ws_f = torch.empty(m.workspace_bytes(shape.T, shape.d_in, shape.d_out, shape.N, shape.r, shape.k, bf),
                       dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(m.gate_backward_workspace_bytes(shape.T, shape.d_in, shape.d_out, shape.N, shape.r, shape.k, bf),
                       dtype=torch.uint8, device="cuda")
    x_in, dy_in = dev["x"].clone(), dev["dy"].clone()

    def step(x, dyt, wsf, wsb):
        out, idx, w = m.linear_forward(x, dev["W"], dev["W_gate"], dev["bias"], dev["A"], dev["B"], shape.k,
                                       shape.scale, ws=wsf, return_routing=True, packed=dev["packed"])
        grads = m.gate_backward(x, dyt, dev["bias"], dev["B"], dev["packed"], shape.k, shape.scale,
                                labels=dev["labels"], beta=0.3, topk_idx=idx, topk_w=w, want_d_logits=True, ws=wsb,
                                forward_ws=wsf, A=dev["A"], W_gate=dev["W_gate"], W_t=W_t, want_dx=True)
        return (out,) + tuple(grads)

    step(x_in, dy_in, ws_f, ws_b)            # first call sets the kernels' LDS attributes
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            held = step(x_in, dy_in, ws_f, ws_b)
    torch.cuda.synchronize()
    gen_t = torch.Generator(device="cuda").manual_seed(6)
    for rep in range(3):
        x_new = torch.randn(x_in.shape, generator=gen_t, device="cuda", dtype=torch.float32).to(bf)
        dy_new = (torch.randn(dy_in.shape, generator=gen_t, device="cuda", dtype=torch.float32) / 16).to(bf)
        ref = step(x_new, dy_new, torch.empty_like(ws_f), torch.empty_like(ws_b))   # eager, own workspaces
        torch.cuda.synchronize()
        x_in.copy_(x_new)
        dy_in.copy_(dy_new)
        for t in held:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("out", "dW_gate", "dbias", "d_logits", "dx"), held, ref):
            assert torch.equal(a, b), f"replay {rep}: {name} differs from the eager call"
