"""Pins for the CPU oracle: it is checked against things other than itself.

* a hand-worked example (tests/golden/hand_example.json; Sec. 3.1, Eq. 2 and Eq. 3),
* a brute-force twin in the per-adapter ("loop-original", Sec. 3.3) form with a
  rank-based one-hot mask, written with numpy matmuls in fp64,
* special cases that reduce to one dense fp64 GEMM (Eq. 1 with a single adapter;
  the average-merge baseline of Sec. 4.1 when all logits tie and k=N),
* invariants of Eq. 2 / Eq. 3 and of the bucketing.

Shapes are deliberately asymmetric (d_in != d_out, r != k, N prime) so that a
transposed operand or a swapped index cannot pass.
"""
import json
import os

import numpy as np
import pytest

import oracle
from gen import inputs as gen

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def _rand_layer(seed, T=7, d_in=12, d_out=20, N=5, r=3, dtype="f32", routing="uniform", k=2):
    shape = gen.LayerShape(T, d_in, d_out, N, r, k, 2.0, dtype, routing, "pin")
    ops = gen.make_layer(shape, seed)
    # O(1) operands so errors are visible
    ops["W_gate"] = ops["W_gate"] * np.float32(np.sqrt(d_in))
    return shape, ops


# ---------------------------------------------------------------- brute force
def brute_force_layer(x, W, W_gate, bias, A, B, k, scale):
    """Per-adapter evaluation: every adapter densely on its token set, one-hot top-k mask."""
    x64, W64 = x.astype(np.float64), W.astype(np.float64)
    g = x64 @ W_gate.astype(np.float64)
    if bias is not None:
        g = g + bias.astype(np.float64)
    g = g.astype(np.float32)
    T, N = g.shape
    # rank of adapter j for token t = number of adapters that beat it
    beats = (g[:, :, None] > g[:, None, :]) | \
            ((g[:, :, None] == g[:, None, :]) & (np.arange(N)[:, None] < np.arange(N)[None, :]))
    rank = beats.sum(axis=1)                    # [T, N]
    mask = rank < k
    g64 = g.astype(np.float64)
    e = np.where(mask, np.exp(g64 - np.where(mask, g64, -np.inf).max(axis=1, keepdims=True)), 0.0)
    w = e / e.sum(axis=1, keepdims=True)        # softmax restricted to the selected k
    y = x64 @ W64.T
    for i in range(N):                          # loop over adapters, gather X_i
        sel = np.nonzero(mask[:, i])[0]
        if sel.size == 0:
            continue
        Xi = x64[sel]
        y[sel] += scale * w[sel, i:i + 1] * ((Xi @ A[i].astype(np.float64)) @ B[i].astype(np.float64))
    return y, g, rank, w


# ------------------------------------------------------------------ the pins
def test_hand_worked_example():
    with open(os.path.join(HERE, "golden", "hand_example.json")) as f:
        ex = json.load(f)
    x, Wg, W = (np.array(ex[n], dtype=np.float32) for n in ("x", "W_gate", "W"))
    A, B = np.array(ex["A"], dtype=np.float32), np.array(ex["B"], dtype=np.float32)
    exp = ex["expect"]
    out = oracle.linear_forward(x, W, Wg, None, A, B, ex["k"], ex["scale"])
    assert np.array_equal(out["logits"], np.array(exp["logits"], dtype=np.float32))
    assert np.array_equal(out["idx"], np.array(exp["idx"]))
    np.testing.assert_allclose(out["w"], exp["w"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(out["y"], exp["y"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(oracle.base(x, W), exp["base"], rtol=0, atol=0)
    _, h = oracle.lora_delta(x, A, B, out["idx"], out["w"], ex["scale"], return_h=True)
    np.testing.assert_allclose(h, exp["h"], rtol=0, atol=0)
    c, o, tok, slot = oracle.bucket(out["idx"], 3)
    assert c.tolist() == exp["counts"] and o.tolist() == exp["offsets"]
    assert tok.tolist() == exp["bucket_tok"] and slot.tolist() == exp["bucket_slot"]


@pytest.mark.parametrize("seed,k,routing", [(0, 1, "uniform"), (1, 2, "uniform"), (2, 3, "zipf"),
                                            (3, 5, "uniform")])
def test_brute_force_twin(seed, k, routing):
    shape, o = _rand_layer(seed, k=k, routing=routing)
    out = oracle.linear_forward(o["x"], o["W"], o["W_gate"], o["bias"], o["A"], o["B"], k, 2.0)
    y, g, rank, w = brute_force_layer(o["x"], o["W"], o["W_gate"], o["bias"], o["A"], o["B"], k, 2.0)
    np.testing.assert_allclose(out["logits"], g, rtol=0, atol=1e-6)
    # selection: adapter idx[t, s] has rank s
    for t in range(shape.T):
        for s in range(k):
            assert rank[t, out["idx"][t, s]] == s
            assert abs(out["w"][t, s] - w[t, out["idx"][t, s]]) < 1e-14
    np.testing.assert_allclose(out["y"], y, rtol=0, atol=1e-11)


def test_row_subset_matches_full():
    shape, o = _rand_layer(4, T=9)
    full = oracle.linear_forward(o["x"], o["W"], o["W_gate"], None, o["A"], o["B"], 2, 2.0)
    rows = np.array([8, 0, 3, 3], dtype=np.int32)
    sub = oracle.linear_forward(o["x"], o["W"], o["W_gate"], None, o["A"], o["B"], 2, 2.0, rows=rows)
    for n in ("y", "logits", "idx", "w"):
        assert np.array_equal(sub[n], full[n][rows])


def test_single_adapter_is_eq1_gemm():
    """N=1, k=1: w=1 and the layer is x(W + s*A*B): one fp64 GEMM (Eq. 1; top-1 remark, App. A.1)."""
    shape, o = _rand_layer(5, N=1, k=1)
    out = oracle.linear_forward(o["x"], o["W"], o["W_gate"], None, o["A"], o["B"], 1, 2.0)
    merged = o["W"].astype(np.float64).T + 2.0 * (o["A"][0].astype(np.float64) @ o["B"][0].astype(np.float64))
    np.testing.assert_allclose(out["y"], o["x"].astype(np.float64) @ merged, rtol=0, atol=1e-12)
    assert np.all(out["w"] == 1.0) and np.all(out["idx"] == 0)


def test_all_tied_full_k_is_average_merge():
    """W_gate=0, k=N: every logit ties, w=1/N, layer = x(W + (s/N) sum A_i B_i) (Avg-Merge, Sec. 4.1)."""
    shape, o = _rand_layer(6, N=5, k=5)
    Wg0 = np.zeros_like(o["W_gate"])
    out = oracle.linear_forward(o["x"], o["W"], Wg0, None, o["A"], o["B"], 5, 2.0)
    assert np.array_equal(out["idx"], np.tile(np.arange(5, dtype=np.int32), (shape.T, 1)))
    np.testing.assert_allclose(out["w"], 0.2, rtol=0, atol=1e-16)
    merged = o["W"].astype(np.float64).T + (2.0 / 5) * sum(
        o["A"][i].astype(np.float64) @ o["B"][i].astype(np.float64) for i in range(5))
    np.testing.assert_allclose(out["y"], o["x"].astype(np.float64) @ merged, rtol=0, atol=1e-12)


def test_zero_B_gives_base_exactly():
    shape, o = _rand_layer(7)
    out = oracle.linear_forward(o["x"], o["W"], o["W_gate"], None, o["A"], np.zeros_like(o["B"]), 2, 2.0)
    assert np.array_equal(out["y"], oracle.base(o["x"], o["W"]))
    np.testing.assert_allclose(out["y"], o["x"].astype(np.float64) @ o["W"].astype(np.float64).T,
                               rtol=0, atol=1e-12)


def test_weights_positive_sum_to_one_and_match_full_softmax():
    shape, o = _rand_layer(8, T=50, N=7, k=3)
    g = oracle.gate_logits(o["x"], o["W_gate"]).astype(np.float32)
    idx, w = oracle.topk_softmax(g, 3)
    assert np.all(w > 0)
    np.testing.assert_allclose(w.sum(axis=1), 1.0, rtol=0, atol=1e-15)
    # softmax over all N, renormalised over the selected k, equals Eq. 3
    g64 = g.astype(np.float64)
    p = np.exp(g64 - g64.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    psel = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    np.testing.assert_allclose(w, psel / psel.sum(axis=1, keepdims=True), rtol=0, atol=1e-14)
    # descending order of the selected logits
    gs = np.take_along_axis(g, idx.astype(np.int64), axis=1)
    assert np.all(gs[:, :-1] >= gs[:, 1:])


def test_topk_matches_stable_argsort_and_tie_break():
    rng = np.random.default_rng(0)
    g = rng.integers(-3, 4, size=(200, 9)).astype(np.float32)      # many exact ties
    for k in (1, 2, 4, 9):
        idx, _ = oracle.topk_softmax(g, k)
        ref = np.argsort(-g, axis=1, kind="stable")[:, :k]          # stable: lower index first
        assert np.array_equal(idx, ref.astype(np.int32))
    # duplicated gate column: identical logits, the lower index must come first
    shape, o = _rand_layer(9, N=5)
    Wg = o["W_gate"].copy()
    Wg[:, 3] = Wg[:, 1]
    gg = oracle.gate_logits(o["x"], Wg).astype(np.float32)
    idx, _ = oracle.topk_softmax(gg, 5)
    for t in range(shape.T):
        pos = idx[t].tolist()
        assert pos.index(1) + 1 == pos.index(3)


def test_gate_logits_match_fp64_matmul_and_bias():
    shape, o = _rand_layer(10, routing="zipf")
    g = oracle.gate_logits(o["x"], o["W_gate"], o["bias"])
    ref = o["x"].astype(np.float64) @ o["W_gate"].astype(np.float64) + o["bias"].astype(np.float64)
    np.testing.assert_allclose(g, ref, rtol=0, atol=1e-13)
    np.testing.assert_allclose(o["bias"], 2 * np.log(1 / (np.arange(5) + 1.0)), rtol=1e-6)


def test_temperature_reading():
    g = np.array([[0.0, 3.0, 1.0]], dtype=np.float32)
    idx, w = oracle.topk_softmax(g, 2, temperature=2.0)
    assert idx.tolist() == [[1, 2]]
    np.testing.assert_allclose(w, [[1 / (1 + np.exp(-1.0)), 1 - 1 / (1 + np.exp(-1.0))]], atol=1e-15)


def test_temperature_in_the_whole_layer():
    """The layer with a temperature: same selection, weights sigma((g0 - g1) / tau) for k = 2 (closed form of a
    two-way softmax), y = base + s * sum w_j * (x A_j) B_j with those weights; tau -> infinity gives the plain mean
    of the k selected adapters; tau = 1 is the untempered layer bit for bit."""
    shape, o = _rand_layer(21, T=9, N=6)
    args = (o["x"], o["W"], o["W_gate"], None, o["A"], o["B"], 2, 2.0)
    ref = oracle.linear_forward(*args)
    one = oracle.linear_forward(*args, temperature=1.0)
    assert np.array_equal(one["y"], ref["y"]) and np.array_equal(one["w"], ref["w"])
    for tau in (15.0, 20.0, 30.0):
        out = oracle.linear_forward(*args, temperature=tau)
        assert np.array_equal(out["idx"], ref["idx"])
        g = ref["logits"].astype(np.float64)
        gap = np.take_along_axis(g, ref["idx"][:, :1].astype(np.int64), 1) - \
            np.take_along_axis(g, ref["idx"][:, 1:2].astype(np.int64), 1)
        w0 = 1.0 / (1.0 + np.exp(-gap / tau))
        np.testing.assert_allclose(out["w"], np.concatenate([w0, 1 - w0], axis=1), rtol=0, atol=1e-15)
        delta = oracle.lora_delta(o["x"], o["A"], o["B"], ref["idx"], out["w"], 2.0)
        np.testing.assert_allclose(out["y"], oracle.base(o["x"], o["W"]) + delta, rtol=0, atol=1e-12)
    far = oracle.linear_forward(*args, temperature=1e12)
    np.testing.assert_allclose(far["w"], 0.5, rtol=0, atol=1e-11)


def test_permutation_invariances():
    shape, o = _rand_layer(11, T=8, N=5)
    ref = oracle.linear_forward(o["x"], o["W"], o["W_gate"], None, o["A"], o["B"], 2, 2.0)
    perm = np.array([3, 0, 4, 1, 2])
    out = oracle.linear_forward(o["x"], o["W"], o["W_gate"][:, perm], None, o["A"][perm], o["B"][perm], 2, 2.0)
    np.testing.assert_allclose(out["y"], ref["y"], rtol=0, atol=1e-12)
    assert np.array_equal(perm[out["idx"]], ref["idx"])
    tperm = np.array([5, 2, 7, 0, 1, 6, 3, 4])
    out = oracle.linear_forward(o["x"][tperm], o["W"], o["W_gate"], None, o["A"], o["B"], 2, 2.0)
    assert np.array_equal(out["y"], ref["y"][tperm])


def test_linear_in_scale_and_top1_ignores_gate_scale():
    shape, o = _rand_layer(12)
    f = lambda s, k=2, wg=o["W_gate"]: oracle.linear_forward(o["x"], o["W"], wg, None, o["A"], o["B"], k, s)["y"]
    y0, y1, y3 = f(0.0), f(1.0), f(3.0)
    np.testing.assert_allclose(y3 - y0, 3 * (y1 - y0), rtol=0, atol=1e-12)
    np.testing.assert_allclose(y0, oracle.base(o["x"], o["W"]), rtol=0, atol=0)
    np.testing.assert_allclose(f(2.0, 1), f(2.0, 1, o["W_gate"] * np.float32(4.0)), rtol=0, atol=0)


def test_lora_delta_matches_per_token_einsum():
    """Eq. 5 (bmm form): entry (t,j) uses A_{I(t)_j}, B_{I(t)_j}, weight w[t,j]; sum over the k entries."""
    shape, o = _rand_layer(13, T=6, N=5, r=3)
    rng = np.random.default_rng(1)
    idx = np.stack([rng.permutation(5)[:2] for _ in range(6)]).astype(np.int32)
    w = rng.random((6, 2))
    delta, h = oracle.lora_delta(o["x"], o["A"], o["B"], idx, w, 1.5, return_h=True)
    A_sel = o["A"].astype(np.float64)[idx]            # [T,k,d,r]   (the gathered copies of bmm-torch)
    B_sel = o["B"].astype(np.float64)[idx]            # [T,k,r,h]
    h_ref = np.einsum("td,tkdr->tkr", o["x"].astype(np.float64), A_sel)
    d_ref = 1.5 * np.einsum("tk,tkr,tkrh->th", w, h_ref, B_sel)
    np.testing.assert_allclose(h, h_ref, rtol=0, atol=1e-13)
    np.testing.assert_allclose(delta, d_ref, rtol=0, atol=1e-12)


def test_bucket_invariants_and_stable_sort():
    rng = np.random.default_rng(2)
    T, k, N = 300, 3, 11
    idx = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
    idx[idx == 4] = 10                                           # make bucket 4 empty (may duplicate 10: allowed here)
    counts, offsets, tok, slot = oracle.bucket(idx, N)
    assert counts.sum() == T * k and counts[4] == 0
    assert offsets[0] == 0 and np.array_equal(offsets[1:], np.cumsum(counts))
    flat = idx.reshape(-1)
    order = np.argsort(flat, kind="stable")                      # library routine: stable sort by adapter
    assert np.array_equal(tok, (order // k).astype(np.int32))
    assert np.array_equal(slot, (order % k).astype(np.int32))
    for j in range(N):
        seg = tok[offsets[j]:offsets[j + 1]]
        assert np.all(np.diff(seg) >= 0)
        assert np.all(idx[seg, slot[offsets[j]:offsets[j + 1]]] == j)


def test_bf16_inputs_are_exact_in_bf16():
    import torch
    shape = gen.LayerShape(5, 64, 32, 3, 4, 2, 2.0, "bf16")
    o = gen.make_layer(shape, 3)
    for n in ("x", "W", "A", "B"):
        t = torch.from_numpy(o[n])
        assert torch.equal(t.to(torch.bfloat16).to(torch.float32), t)
    raw = gen.make_layer(gen.LayerShape(5, 64, 32, 3, 4, 2, 2.0, "f32"), 3)["x"]
    assert torch.equal(torch.from_numpy(raw).to(torch.bfloat16).to(torch.float32), torch.from_numpy(o["x"]))


def test_margin_conditioning_removes_near_ties():
    from oracle import margin
    seed, layers = gen.config_layers(1)
    shape = gen.LayerShape(2000, 64, 64, 28, 8, 2, 2.0, "bf16")
    o = gen.make_layer(shape, seed, only=("x", "W_gate"))
    before = margin.small_margin_rows(oracle.gate_logits(o["x"], o["W_gate"]), 2, 1e-3)
    n = margin.condition_margins(shape, seed, 0, o["x"], o["W_gate"], None, 1e-3)
    after = margin.small_margin_rows(oracle.gate_logits(o["x"], o["W_gate"]), 2, 1e-3)
    assert n >= before.size and after.size == 0
    # deterministic
    o2 = gen.make_layer(shape, seed, only=("x", "W_gate"))
    margin.condition_margins(shape, seed, 0, o2["x"], o2["W_gate"], None, 1e-3)
    assert np.array_equal(o["x"], o2["x"])


# ------------------------------------------------- gate gradients (Sec. 3.2, Eq. 4)
def _loss_of_gate(ops, W_gate, bias, dy, idx, k, scale, labels, beta, x=None):
    """The scalar that the gate gradients differentiate, built from the forward definitions only:
    <dy, o> with o from Eq. 2 (selection idx held fixed, weights from Eq. 3 on the k selected logits in
    double) plus beta * sum_t cross-entropy(softmax over all N logits, label_t)."""
    xx = ops["x"] if x is None else x
    x64 = xx.astype(np.float64)
    g = x64 @ W_gate + bias
    gs = np.take_along_axis(g, idx.astype(np.int64), axis=1)
    e = np.exp(gs - gs.max(axis=1, keepdims=True))
    w = e / e.sum(axis=1, keepdims=True)
    if x is None:
        y = oracle.base(ops["x"], ops["W"]) + oracle.lora_delta(ops["x"], ops["A"], ops["B"], idx, w, scale)
    else:   # the C oracle takes float32 inputs; a probe of x needs double: Eq. 2 written out with numpy here
        y = x64 @ ops["W"].astype(np.float64).T
        for t in range(x64.shape[0]):
            for j in range(k):
                a = idx[t, j]
                y[t] += scale * w[t, j] * ((x64[t] @ ops["A"][a].astype(np.float64)) @ ops["B"][a].astype(np.float64))
    loss = float((dy * y).sum())
    if beta:
        lse = np.log(np.exp(g - g.max(axis=1, keepdims=True)).sum(axis=1)) + g.max(axis=1)
        loss += beta * float((lse - g[np.arange(g.shape[0]), labels]).sum())
    return loss


def _backward_case(seed, k, T=6, d_in=10, d_out=14, N=5, r=3):
    from oracle import gate_backward as gb
    shape, ops = _rand_layer(seed, T=T, d_in=d_in, d_out=d_out, N=N, r=r, k=k)
    rng = np.random.default_rng(seed + 100)
    dy = rng.standard_normal((T, d_out))
    labels = rng.integers(0, N, size=T)
    bias = rng.standard_normal(N).astype(np.float32) * np.float32(0.3)
    return gb, shape, ops, dy, labels, bias


@pytest.mark.parametrize("k", [1, 2, 3, 5])
@pytest.mark.parametrize("beta", [0.0, 0.7])
def test_gate_backward_matches_finite_differences_of_the_forward(k, beta):
    gb, shape, ops, dy, labels, bias = _backward_case(31 + k, k)
    res = gb.gate_backward(ops["x"], dy, ops["W_gate"], bias, ops["A"], ops["B"], k, shape.scale, labels, beta)
    # the selection must not change under the probes below: every gap among ranks 1..k+1 is far above them
    g = oracle.gate_logits(ops["x"], ops["W_gate"], bias)
    top = -np.sort(-g, axis=1)[:, :min(k + 1, g.shape[1])]
    assert (top[:, :-1] - top[:, 1:]).min() > 1e-3
    Wg64, b64 = ops["W_gate"].astype(np.float64), bias.astype(np.float64)
    eps = 1e-6
    rng = np.random.default_rng(5)
    for _ in range(12):
        i, n = int(rng.integers(0, Wg64.shape[0])), int(rng.integers(0, Wg64.shape[1]))
        Wp, Wm = Wg64.copy(), Wg64.copy()
        Wp[i, n] += eps
        Wm[i, n] -= eps
        fd = (_loss_of_gate(ops, Wp, b64, dy, res["idx"], k, shape.scale, labels, beta) -
              _loss_of_gate(ops, Wm, b64, dy, res["idx"], k, shape.scale, labels, beta)) / (2 * eps)
        assert abs(fd - res["dW_gate"][i, n]) <= 1e-5 * max(1.0, abs(fd)), (i, n, fd, res["dW_gate"][i, n])
    for n in range(b64.size):
        bp, bm = b64.copy(), b64.copy()
        bp[n] += eps
        bm[n] -= eps
        fd = (_loss_of_gate(ops, Wg64, bp, dy, res["idx"], k, shape.scale, labels, beta) -
              _loss_of_gate(ops, Wg64, bm, dy, res["idx"], k, shape.scale, labels, beta)) / (2 * eps)
        assert abs(fd - res["dbias"][n]) <= 1e-5 * max(1.0, abs(fd)), (n, fd, res["dbias"][n])


def test_gate_backward_top1_has_no_language_model_part():
    """App. "Top-1 strategy": with k = 1 the weight is the constant 1, the output does not depend on the gate,
    so only the classification loss reaches it; with beta = 0 every gradient is exactly zero."""
    gb, shape, ops, dy, labels, bias = _backward_case(41, 1)
    res = gb.gate_backward(ops["x"], dy, ops["W_gate"], bias, ops["A"], ops["B"], 1, shape.scale, labels, 0.0)
    assert not res["dW_gate"].any() and not res["dbias"].any()
    res = gb.gate_backward(ops["x"], dy, ops["W_gate"], bias, ops["A"], ops["B"], 1, shape.scale, labels, 0.5)
    g = oracle.gate_logits(ops["x"], ops["W_gate"], bias).astype(np.float32).astype(np.float64)
    p = np.exp(g - g.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    p[np.arange(len(labels)), labels] -= 1.0
    np.testing.assert_allclose(res["d_logits"], 0.5 * p, rtol=0, atol=1e-14)


@pytest.mark.parametrize("k", [2, 4])
def test_gate_backward_invariants(k):
    """Both softmaxes are shift invariant, so each token's logit gradient sums to zero; unselected adapters get
    only the classification part; dW_gate is the outer-product sum of x and d_logits."""
    gb, shape, ops, dy, labels, bias = _backward_case(51 + k, k)
    res = gb.gate_backward(ops["x"], dy, ops["W_gate"], bias, ops["A"], ops["B"], k, shape.scale, labels, 0.3)
    assert np.abs(res["d_logits"].sum(axis=1)).max() < 1e-12
    assert np.abs(res["dbias"].sum()) < 1e-12
    lm_only = gb.gate_backward(ops["x"], dy, ops["W_gate"], bias, ops["A"], ops["B"], k, shape.scale, None, 0.0)
    sel = np.zeros_like(lm_only["d_logits"], dtype=bool)
    np.put_along_axis(sel, lm_only["idx"].astype(np.int64), True, axis=1)
    assert not lm_only["d_logits"][~sel].any()
    acc = np.zeros_like(res["dW_gate"])
    for t in range(ops["x"].shape[0]):
        acc += np.outer(ops["x"][t].astype(np.float64), res["d_logits"][t])
    np.testing.assert_allclose(res["dW_gate"], acc, rtol=1e-12, atol=1e-12)
    # scaling dy scales the language-model part linearly
    twice = gb.gate_backward(ops["x"], 2 * dy, ops["W_gate"], bias, ops["A"], ops["B"], k, shape.scale, None, 0.0)
    np.testing.assert_allclose(twice["dW_gate"], 2 * lm_only["dW_gate"], rtol=1e-12, atol=1e-12)


def test_gate_backward_unlabelled_tokens_have_no_classification_part():
    gb, shape, ops, dy, labels, bias = _backward_case(61, 2)
    lab = labels.copy()
    lab[1], lab[4] = -1, 99
    res = gb.gate_backward(ops["x"], dy, ops["W_gate"], bias, ops["A"], ops["B"], 2, shape.scale, lab, 0.4)
    lm = gb.gate_backward(ops["x"], dy, ops["W_gate"], bias, ops["A"], ops["B"], 2, shape.scale, None, 0.0)
    full = gb.gate_backward(ops["x"], dy, ops["W_gate"], bias, ops["A"], ops["B"], 2, shape.scale, labels, 0.4)
    for t in range(len(lab)):
        want = lm if t in (1, 4) else full
        np.testing.assert_array_equal(res["d_logits"][t], want["d_logits"][t])


@pytest.mark.parametrize("k", [1, 2, 4])
def test_gate_backward_dx_matches_finite_differences_of_the_forward(k):
    """dx collects the base projection, the selected adapters and the gate: central differences of the same
    loss with respect to entries of x (in double; Eq. 2 in numpy agrees with the C oracle at the unperturbed x)."""
    gb, shape, ops, dy, labels, bias = _backward_case(71 + k, k)
    beta = 0.6
    res = gb.gate_backward(ops["x"], dy, ops["W_gate"], bias, ops["A"], ops["B"], k, shape.scale, labels, beta,
                           W=ops["W"])
    Wg64, b64 = ops["W_gate"].astype(np.float64), bias.astype(np.float64)
    x64 = ops["x"].astype(np.float64)
    base = _loss_of_gate(ops, Wg64, b64, dy, res["idx"], k, shape.scale, labels, beta)
    twin = _loss_of_gate(ops, Wg64, b64, dy, res["idx"], k, shape.scale, labels, beta, x=x64)
    assert abs(base - twin) <= 1e-9 * max(1.0, abs(base))
    eps = 1e-6
    rng = np.random.default_rng(9)
    for _ in range(16):
        t, i = int(rng.integers(0, x64.shape[0])), int(rng.integers(0, x64.shape[1]))
        xp, xm = x64.copy(), x64.copy()
        xp[t, i] += eps
        xm[t, i] -= eps
        fd = (_loss_of_gate(ops, Wg64, b64, dy, res["idx"], k, shape.scale, labels, beta, x=xp) -
              _loss_of_gate(ops, Wg64, b64, dy, res["idx"], k, shape.scale, labels, beta, x=xm)) / (2 * eps)
        assert abs(fd - res["dx"][t, i]) <= 1e-5 * max(1.0, abs(fd)), (t, i, fd, res["dx"][t, i])
    # without adapters' weight and gate (scale 0, beta 0) dx is the base projection's: dy W
    plain = gb.gate_backward(ops["x"], dy, ops["W_gate"], bias, ops["A"], ops["B"], k, 0.0, None, 0.0, W=ops["W"])
    np.testing.assert_allclose(plain["dx"], dy @ ops["W"].astype(np.float64), rtol=1e-12, atol=1e-12)


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """Host sanitizer build of the checker: the C oracle compiled with -fsanitize=address,undefined runs the
    hand-worked example, a ragged row subset and a layer of rank 300 (beyond any fixed buffer) in a child process
    without a report.  The sanitizer runtime has to be loaded first, hence the child process and LD_PRELOAD."""
    import subprocess
    import sys
    import textwrap
    src = os.path.join(ROOT, "oracle", "meteora_oracle.c")
    lib = str(tmp_path / "liboracle_asan.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c99", "-fPIC", "-shared", "-fno-omit-frame-pointer",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-ffp-contract=off",
                           "-o", lib, src, "-lm"])
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    ubsan = subprocess.check_output(["gcc", "-print-file-name=libubsan.so"], text=True).strip()
    code = textwrap.dedent(f"""
        import ctypes, json, numpy as np
        L = ctypes.CDLL({lib!r})
        ex = json.load(open({os.path.join(ROOT, "tests", "golden", "hand_example.json")!r}))
        f = lambda a: np.ascontiguousarray(a, dtype=np.float32)
        p = lambda a: a.ctypes.data_as(ctypes.c_void_p)
        def layer(x, W, Wg, A, B, k, scale, rows=None):
            T, d_in = x.shape; d_out = W.shape[0]; N, _, r = A.shape
            n = T if rows is None else rows.size
            y = np.empty((n, d_out)); lg = np.empty((n, N), dtype=np.float32)
            idx = np.empty((n, k), dtype=np.int32); w = np.empty((n, k))
            s64 = np.empty((n, N)); dl = np.empty((n, d_out))
            L.oracle_linear_forward(p(x), p(W), p(Wg), None, p(A), p(B), ctypes.c_int(d_in), ctypes.c_int(d_out),
                                    ctypes.c_int(N), ctypes.c_int(r), ctypes.c_int(k), ctypes.c_double(scale),
                                    ctypes.c_double(1.0), None if rows is None else p(rows), ctypes.c_int(n), p(y),
                                    p(lg), p(idx), p(w), p(s64), p(dl))
            return y, idx
        y, idx = layer(f(ex["x"]), f(ex["W"]), f(ex["W_gate"]), f(ex["A"]), f(ex["B"]), ex["k"], ex["scale"])
        assert np.allclose(y, ex["expect"]["y"], atol=1e-12) and idx.tolist() == ex["expect"]["idx"]
        g = np.random.default_rng(0)
        T, d_in, d_out, N, r = 11, 9, 13, 4, 300
        x, W, Wg = f(g.standard_normal((T, d_in))), f(g.standard_normal((d_out, d_in))), f(g.standard_normal((d_in, N)))
        A, B = f(g.standard_normal((N, d_in, r))), f(g.standard_normal((N, r, d_out)))
        rows = np.array([10, 0, 3], dtype=np.int32)
        y, idx = layer(x, W, Wg, A, B, 3, 0.5, rows)
        tok = np.array([[0, 1, 0], [2, 2, 1]], dtype=np.int32)      # bucketing with an empty bucket
        c = np.empty(4, dtype=np.int32); o = np.empty(5, dtype=np.int32)
        bt = np.empty(6, dtype=np.int32); bs = np.empty(6, dtype=np.int32)
        L.oracle_bucket(p(tok), ctypes.c_int(2), ctypes.c_int(3), ctypes.c_int(4), p(c), p(o), p(bt), p(bs))
        assert c.tolist() == [2, 2, 2, 0]
        print("sanitized oracle ok")
    """)
    # the sanitizer runtimes go first; whatever the environment already preloads stays in the list
    preload = " ".join([asan, ubsan, os.environ.get("LD_PRELOAD", "")]).strip()
    env = dict(os.environ, LD_PRELOAD=preload, ASAN_OPTIONS="detect_leaks=0", OMP_NUM_THREADS="2")
    res = subprocess.run([sys.executable, "-c", code], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                         text=True, timeout=300)
    assert res.returncode == 0 and "sanitized oracle ok" in res.stdout, res.stdout[-3000:]
