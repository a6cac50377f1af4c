"""GPU parity: the HIP library, called through its C ABI (ctypes binding), against the CPU oracle.

Bars: routing (top-k indices) and bucketing bit-exact; gate weights within 1e-6; outputs within
max|y - y_ref| / max|y_ref| <= 5e-3 (bf16 storage, fp32 accumulation) or 1e-5 (fp32).
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import margin
import paper_2405_13053_amd as m
from gen import inputs as gen
from tests import util

pytestmark = pytest.mark.gpu

LS = gen.LayerShape


def _np(t):
    return t.detach().cpu().numpy()


# ------------------------------------------------------------------------------ gate / routing
GATE_SHAPES = [
    LS(64, 256, 256, 4, 8, 2, 2.0, "f32", "uniform", "cfg1"),
    LS(257, 1024, 64, 28, 8, 2, 2.0, "bf16", "uniform", "ragged-T"),
    LS(1000, 4096, 64, 28, 8, 2, 2.0, "bf16", "zipf", "zipf"),
    LS(130, 520, 64, 37, 8, 3, 2.0, "bf16", "uniform", "N>32,odd-K"),
    LS(96, 5120, 64, 64, 8, 8, 2.0, "bf16", "uniform", "N=64,k=8"),
    LS(33, 264, 64, 5, 8, 1, 2.0, "f32", "zipf", "top1"),
    LS(1, 4096, 64, 28, 8, 2, 2.0, "bf16", "uniform", "T=1"),
]


@pytest.mark.parametrize("shape", GATE_SHAPES, ids=lambda s: s.name)
def test_gate_topk_matches_oracle(shape):
    ops, dev = util.make_case(shape, seed=11)
    g64, g32, idx_ref, w_ref = util.oracle_routing(ops, shape.k)
    idx, w, logits = m.gate_topk(dev["x"], dev["W_gate"], dev["bias"], shape.k, want_logits=True)
    torch.cuda.synchronize()
    idx, w, logits = _np(idx), _np(w), _np(logits)
    # (1) logit accuracy: fp32 accumulation noise, scaled by the sum of |terms|
    mag = np.abs(ops["x"].astype(np.float64)) @ np.abs(ops["W_gate"].astype(np.float64))
    if ops["bias"] is not None:
        mag = mag + np.abs(ops["bias"].astype(np.float64))
    assert np.all(np.abs(logits - g64) <= 8 * 2.0 ** -24 * mag + 1e-30)
    # (2) selection logic on the GPU's own logits: zero tolerance
    idx_self, w_self = oracle.topk_softmax(logits, shape.k)
    assert np.array_equal(idx, idx_self)
    np.testing.assert_allclose(w, w_self, rtol=0, atol=1e-6)
    # (3) routing equals the oracle's, bit-exact (inputs are margin-conditioned)
    assert np.array_equal(idx, idx_ref)
    # (4) Eq. 3 weights vs the oracle's: d(softmax)/d(logit) <= 1/4 per logit, so the logit noise of (1)
    #     moves a weight by at most half the largest logit deviation, on top of the 1e-6 of (2)
    np.testing.assert_allclose(w, w_ref, rtol=0, atol=1e-6 + 0.5 * float(np.abs(logits - g32).max()))
    np.testing.assert_allclose(w.sum(axis=1), 1.0, rtol=0, atol=1e-6)
    assert np.all(w > 0)


def test_gate_selection_logic_on_unconditioned_inputs():
    """Near ties are allowed to resolve either way vs. fp64, but never against the GPU's own logits."""
    shape = LS(3000, 512, 64, 28, 8, 2, 2.0, "bf16")
    ops, dev = util.make_case(shape, seed=5, condition=False)
    idx, w, logits = m.gate_topk(dev["x"], dev["W_gate"], None, 2, want_logits=True)
    idx_self, _ = oracle.topk_softmax(_np(logits), 2)
    assert np.array_equal(_np(idx), idx_self)


def test_gate_exact_ties_lowest_index_first():
    shape = LS(200, 512, 64, 12, 8, 4, 2.0, "bf16")
    ops, dev = util.make_case(shape, seed=6, condition=False)
    Wg = ops["W_gate"].copy()
    Wg[:, 7] = Wg[:, 2]          # identical columns -> bit-identical logits in any summation order
    Wg[:, 9] = Wg[:, 2]
    idx, w, logits = m.gate_topk(dev["x"], util.to_dev(Wg, torch.float32), None, 4, want_logits=True)
    logits = _np(logits)
    assert np.array_equal(logits[:, 2], logits[:, 7]) and np.array_equal(logits[:, 2], logits[:, 9])
    idx_self, _ = oracle.topk_softmax(logits, 4)
    assert np.array_equal(_np(idx), idx_self)
    # all-zero gate with k = N: every logit ties, order is 0..N-1 and w = 1/N
    z = torch.zeros((512, 12), dtype=torch.float32, device="cuda")
    idx, w, _ = m.gate_topk(dev["x"], z, None, 8)
    assert np.array_equal(_np(idx), np.tile(np.arange(8, dtype=np.int32), (200, 1)))
    np.testing.assert_allclose(_np(w), 1.0 / 8, rtol=0, atol=1e-7)


def test_gate_temperature():
    shape = LS(100, 256, 64, 6, 8, 2, 2.0, "f32")
    ops, dev = util.make_case(shape, seed=7)
    idx, w, logits = m.gate_topk(dev["x"], dev["W_gate"], None, 2, inv_temperature=1 / 15.0, want_logits=True)
    idx_ref, w_ref = oracle.topk_softmax(_np(logits), 2, temperature=15.0)
    assert np.array_equal(_np(idx), idx_ref)
    np.testing.assert_allclose(_np(w), w_ref, rtol=0, atol=1e-6)


# ------------------------------------------------------------------------------------ bucketing
@pytest.mark.parametrize("T,k,N,mode", [(64, 2, 4, "uniform"), (4096, 2, 28, "uniform"), (8192, 2, 28, "zipf"),
                                        (1023, 3, 64, "uniform"), (513, 1, 7, "one-bucket"), (1, 2, 28, "uniform"),
                                        (16384, 2, 28, "zipf"), (700, 8, 9, "uniform")])
def test_bucket_tokens_bit_exact(T, k, N, mode):
    rng = np.random.default_rng(T * 131 + k)
    if mode == "one-bucket":
        idx = np.full((T, k), 3, dtype=np.int32)
    else:
        # k distinct adapters per token, drawn with probabilities p (Gumbel top-k)
        p = 1.0 / (np.arange(N) + 1.0) ** 2 if mode == "zipf" else np.ones(N)
        scores = np.log(p)[None, :] + rng.gumbel(size=(T, N))
        idx = np.argsort(-scores, axis=1)[:, :k].astype(np.int32)
    c_ref, o_ref, tok_ref, slot_ref = oracle.bucket(idx, N)
    c, o, tok, slot = m.bucket_tokens(torch.from_numpy(idx).cuda(), N)
    assert np.array_equal(_np(c), c_ref)
    assert np.array_equal(_np(o), o_ref)
    assert np.array_equal(_np(tok), tok_ref)
    assert np.array_equal(_np(slot), slot_ref)
    assert int(_np(c).sum()) == T * k


# ------------------------------------------------------------------------------------ LoRA term
LORA_SHAPES = [
    LS(64, 256, 256, 4, 8, 2, 2.0, "f32", "uniform", "cfg1"),
    LS(300, 512, 1032, 28, 8, 2, 2.0, "bf16", "uniform", "bf16-r8"),
    LS(517, 1024, 520, 28, 16, 2, 2.0, "bf16", "zipf", "bf16-r16-zipf"),
    LS(70, 264, 136, 6, 5, 3, 0.5, "bf16", "uniform", "odd-r"),
    LS(40, 128, 64, 3, 64, 1, 1.0, "f32", "uniform", "r64-top1"),
    # >= 16384 (token, slot) pairs: the shrink runs whole-K tiles and the scatter clears the expand operand
    LS(8300, 520, 136, 28, 16, 2, 2.0, "bf16", "zipf", "whole-K-shrink-ragged"),
    LS(4200, 264, 72, 5, 40, 4, 1.0, "bf16", "uniform", "whole-K-shrink-r40"),
]


@pytest.mark.parametrize("shape", LORA_SHAPES, ids=lambda s: s.name)
def test_lora_forward_matches_oracle(shape):
    ops, dev = util.make_case(shape, seed=21)
    _, _, idx_ref, w_ref = util.oracle_routing(ops, shape.k)
    delta_ref = oracle.lora_delta(ops["x"], ops["A"], ops["B"], idx_ref, w_ref, shape.scale)
    idx_d = torch.from_numpy(idx_ref).cuda()
    w_d = torch.from_numpy(w_ref.astype(np.float32)).cuda()
    out = m.lora_forward(dev["x"], dev["A"], dev["B"], idx_d, w_d, shape.scale)
    assert util.rel_max_err(out, delta_ref) <= util.tol(shape)
    # accumulate=1 on top of the base projection
    base_ref = oracle.base(ops["x"], ops["W"])
    out2 = util.to_dev(base_ref.astype(np.float32), util.torch_dtype(shape))
    base_stored = out2.to(torch.float64).cpu().numpy()
    m.lora_forward(dev["x"], dev["A"], dev["B"], idx_d, w_d, shape.scale, out=out2, accumulate=True)
    assert util.rel_max_err(out2, base_stored + delta_ref) <= util.tol(shape)


# --------------------------------------------------------------------------------- base GEMM
@pytest.mark.parametrize("T,d_in,d_out,dtype", [(64, 256, 256, "f32"), (300, 520, 264, "bf16"),
                                                (1024, 1024, 1024, "bf16"), (17, 4096, 72, "bf16"),
                                                (1300, 192, 4104, "bf16"),      # 256 x 128 tiles, ragged both ways
                                                (2600, 128, 4104, "bf16"),      # 256 x 256 tiles, ragged both ways
                                                (4400, 128, 4104, "bf16")])     # 306 big tiles: 128 x 128 tiles instead
def test_base_gemm_matches_oracle(T, d_in, d_out, dtype):
    shape = LS(T, d_in, d_out, 2, 2, 1, 1.0, dtype)
    ops, dev = util.make_case(shape, seed=31, condition=False)
    out = m.base_gemm(dev["x"], dev["W"])
    assert util.rel_max_err(out, oracle.base(ops["x"], ops["W"])) <= util.tol(shape)


# --------------------------------------------------------------------------------- whole layer
LAYER_SHAPES = [
    LS(64, 256, 256, 4, 8, 2, 2.0, "f32", "uniform", "cfg1"),
    LS(333, 512, 776, 28, 8, 2, 2.0, "bf16", "uniform", "bf16-ragged"),
    LS(512, 1024, 512, 28, 16, 2, 2.0, "bf16", "zipf", "bf16-r16-zipf"),
    LS(50, 264, 136, 7, 5, 3, 1.5, "f32", "uniform", "f32-odd"),
    LS(100, 512, 256, 28, 8, 1, 2.0, "bf16", "uniform", "top1"),
]


def _check_layer(shape, seed, layer=0, rows="all", inv_temperature=1.0):
    ops, dev = util.make_case(shape, seed, layer)
    g64 = oracle.gate_logits(ops["x"], ops["W_gate"], ops["bias"])
    g32 = g64.astype(np.float32)
    idx_ref, w_ref = oracle.topk_softmax(g32, shape.k, temperature=1.0 / inv_temperature)
    out, idx, w = m.linear_forward(dev["x"], dev["W"], dev["W_gate"], dev["bias"], dev["A"], dev["B"], shape.k,
                                   shape.scale, return_routing=True, inv_temperature=inv_temperature)
    torch.cuda.synchronize()
    assert np.array_equal(_np(idx), idx_ref), "routing differs from the oracle"
    assert np.all(np.abs(_np(w) - w_ref) <= util.weight_bound(ops, idx_ref, inv_temperature)), "gate weights off"
    if rows == "all":
        sel = None
        y_gpu = out
    else:
        c, o, tok, _ = oracle.bucket(idx_ref, shape.N)
        sel = util.sample_rows(shape.T, c, o, tok)
        y_gpu = out[torch.from_numpy(sel.astype(np.int64)).cuda()]
    ref = oracle.linear_forward(ops["x"], ops["W"], ops["W_gate"], ops["bias"], ops["A"], ops["B"], shape.k,
                                shape.scale, rows=sel, temperature=1.0 / inv_temperature)
    err = util.rel_max_err(y_gpu, ref["y"])
    assert err <= util.tol(shape), f"{shape.name}: rel err {err:.3e}"
    # weights packed once (meteora_pack_weights) instead of per call: the same kernels on the same layouts
    packed = m.pack_weights(dev["W_gate"], dev["A"], dev["B"])
    out_p, idx_p, w_p = m.linear_forward(dev["x"], dev["W"], dev["W_gate"], dev["bias"], dev["A"], dev["B"],
                                         shape.k, shape.scale, return_routing=True, packed=packed,
                                         inv_temperature=inv_temperature)
    assert torch.equal(out_p, out) and torch.equal(idx_p, idx) and torch.equal(w_p, w)
    return out


@pytest.mark.parametrize("shape", LAYER_SHAPES, ids=lambda s: s.name)
def test_linear_forward_matches_oracle(shape):
    _check_layer(shape, seed=41)


@pytest.mark.parametrize("d_in,same_kernel", [(128, True), (512, False)])
def test_linear_forward_zero_B_is_base_and_deterministic(d_in, same_kernel):
    """B = 0: the layer is the base projection.  d_in = 128: the same GEMM kernel as meteora_base_gemm runs, equal
    bits; d_in = 512: this batch's projection is split along K (other fp32 summation order than the one-sweep
    base GEMM), so the bf16 results agree up to the rounding of sums that differ in their last bits."""
    shape = LS(200, d_in, 520, 28, 8, 2, 2.0, "bf16")
    ops, dev = util.make_case(shape, seed=42)
    zB = torch.zeros_like(dev["B"])
    y0 = m.linear_forward(dev["x"], dev["W"], dev["W_gate"], None, dev["A"], zB, 2, 2.0)
    yb = m.base_gemm(dev["x"], dev["W"])
    if same_kernel:
        assert torch.equal(y0, yb)
    else:
        diff = (y0.float() - yb.float()).abs()
        assert float((diff / yb.float().abs().clamp_min(1e-3)).max()) <= 2.0 ** -7      # one bf16 ulp
        assert float((diff > 0).float().mean()) <= 0.02
    y1 = m.linear_forward(dev["x"], dev["W"], dev["W_gate"], None, dev["A"], dev["B"], 2, 2.0)
    y2 = m.linear_forward(dev["x"], dev["W"], dev["W_gate"], None, dev["A"], dev["B"], 2, 2.0)
    assert torch.equal(y1, y2)


def test_packed_weights_serve_many_batches():
    """One blob, two different batches and batch sizes: each equals the per-call-packing result."""
    shape = LS(333, 1024, 776, 28, 8, 2, 2.0, "bf16")
    ops, dev = util.make_case(shape, seed=44)
    packed = m.pack_weights(dev["W_gate"], dev["A"], dev["B"])
    assert packed.numel() == m.packed_bytes(1024, 776, 28, 8, "bf16")
    for rows in (slice(0, 333), slice(17, 150)):
        x = dev["x"][rows].contiguous()
        y_ref = m.linear_forward(x, dev["W"], dev["W_gate"], None, dev["A"], dev["B"], 2, 2.0)
        y = m.linear_forward(x, dev["W"], dev["W_gate"], None, dev["A"], dev["B"], 2, 2.0, packed=packed)
        assert torch.equal(y, y_ref)


SMALL_BATCH_SHAPES = [
    LS(1, 512, 256, 28, 8, 2, 2.0, "bf16", "uniform", "T=1"),
    LS(64, 1024, 776, 12, 16, 3, 1.5, "bf16", "zipf", "T=64-r16-k3-bias-two-launch"),
    LS(40, 4096, 1032, 28, 8, 2, 2.0, "bf16", "uniform", "T=40-ragged-tiles"),
    LS(7, 264, 136, 5, 16, 1, 1.0, "bf16", "zipf", "T=7-r16-top1-ragged"),
    LS(64, 1024, 520, 64, 32, 8, 0.5, "bf16", "uniform", "T=64-N64-r32-k8"),
    LS(33, 5120, 264, 28, 8, 2, 2.0, "bf16", "zipf", "T=33-decode-shape"),
    LS(48, 1024, 520, 28, 16, 2, 2.0, "bf16", "uniform", "T=48-r16-N28-two-launch"),
    # the decode tail's loops: k*r = 256 shrink values per token (four groups of 64 / r slots), a row of 513
    # 8-column pieces (nine stretches, the last with one active lane), top-1
    LS(50, 1024, 776, 16, 32, 8, 0.5, "bf16", "zipf", "T=50-N16-r32-k8-tail"),
    LS(9, 1024, 4104, 28, 8, 8, 1.0, "bf16", "uniform", "T=9-k8-ragged-stretch"),
    LS(64, 2048, 1544, 28, 8, 1, 2.0, "bf16", "zipf", "T=64-top1-tail"),
]


@pytest.mark.parametrize("shape", SMALL_BATCH_SHAPES, ids=lambda s: s.name)
def test_small_batch_path_matches_oracle_and_gate_entry_point(shape):
    """T <= 64: top-k and shrink run token-major in one launch; same adapters as meteora_gate_topk picks."""
    out = _check_layer(shape, seed=45)
    ops, dev = util.make_case(shape, seed=45)
    _, idx, w = m.linear_forward(dev["x"], dev["W"], dev["W_gate"], dev["bias"], dev["A"], dev["B"], shape.k,
                                 shape.scale, return_routing=True)
    idx_g, w_g, _ = m.gate_topk(dev["x"], dev["W_gate"], dev["bias"], shape.k)
    assert torch.equal(idx, idx_g)
    # where the logits come out of the GEMM's own launch they are summed in another order than the gate kernel's
    assert float((w - w_g).abs().max()) <= 1e-5
    # and the LoRA term alone through the bucketed path gives the same layer output to bf16 accuracy
    base = m.base_gemm(dev["x"], dev["W"])
    full = m.lora_forward(dev["x"], dev["A"], dev["B"], idx, w, shape.scale, out=base.clone(), accumulate=True)
    assert util.rel_max_err(full, out.to(torch.float64).cpu().numpy()) <= 2 * util.tol(shape)


# mid-sized batches (64 < T <= 8192, bf16, r % 8 == 0, d_in % 64 == 0, 96 + N*r <= 320): gate logits and the shrink
# of every adapter in one MFMA launch, selection afterwards; 128x128 tiles up to 4096 tokens, 128x320 above
DENSE_ROUTE_SHAPES = [
    LS(65, 64, 72, 3, 8, 1, 2.0, "bf16", "uniform", "T=65-one-K-tile"),
    LS(129, 320, 264, 9, 24, 4, 0.7, "bf16", "zipf", "T=129-r24-k4-bias"),
    LS(1000, 1088, 520, 28, 8, 2, 2.0, "bf16", "zipf", "T=1000-ragged-K17"),
    LS(700, 512, 256, 7, 32, 7, 1.0, "bf16", "uniform", "T=700-r32-k=N"),
    LS(4097, 256, 136, 28, 8, 2, 2.0, "bf16", "uniform", "T=4097-wide-tiles"),
    LS(5000, 832, 264, 14, 16, 3, 2.0, "bf16", "zipf", "T=5000-r16-wide-tiles"),
    LS(260, 384, 136, 28, 8, 8, 1.0, "bf16", "uniform", "T=260-k8"),
    # few output tiles: the base projection is split along K and the expand runs inside the reduction
    LS(256, 4096, 4096, 28, 8, 2, 2.0, "bf16", "uniform", "T=256-split-K-projection"),
    LS(200, 1024, 1096, 28, 8, 2, 2.0, "bf16", "zipf", "T=200-split-K-ragged-columns"),
    LS(513, 2048, 520, 7, 32, 3, 0.5, "bf16", "uniform", "T=513-split-K-r32"),
    # the split projection has more K splits (8) than the routing products alone would take (5)
    LS(3000, 4096, 256, 28, 8, 2, 2.0, "bf16", "uniform", "T=3000-narrow-output-more-splits"),
    # 28 adapters of rank 16: 544 rows of Wcat, several column tiles of the routing products
    LS(70, 512, 264, 28, 16, 2, 2.0, "bf16", "zipf", "T=70-r16-N28-split-K"),
    LS(1000, 1088, 520, 28, 16, 2, 2.0, "bf16", "uniform", "T=1000-r16-N28"),
    LS(4500, 256, 136, 28, 16, 3, 2.0, "bf16", "zipf", "T=4500-r16-N28-two-wide-tiles"),
    LS(300, 320, 200, 32, 16, 4, 1.0, "bf16", "uniform", "T=300-r16-N32-608-rows"),
]


@pytest.mark.parametrize("shape", DENSE_ROUTE_SHAPES, ids=lambda s: s.name)
def test_dense_route_path_matches_oracle_and_bucketed_path(shape):
    """Same routing as meteora_gate_topk bit for bit; the layer equals base GEMM + bucketed LoRA to bf16 accuracy."""
    rows = "all" if shape.T <= 1000 else "sample"
    out = _check_layer(shape, seed=46, rows=rows)
    ops, dev = util.make_case(shape, seed=46)
    _, idx, w = m.linear_forward(dev["x"], dev["W"], dev["W_gate"], dev["bias"], dev["A"], dev["B"], shape.k,
                                 shape.scale, return_routing=True)
    idx_g, w_g, _ = m.gate_topk(dev["x"], dev["W_gate"], dev["bias"], shape.k)
    assert torch.equal(idx, idx_g)
    assert float((w - w_g).abs().max()) <= 1e-5     # the two paths add the logit terms in different orders
    base = m.base_gemm(dev["x"], dev["W"])
    full = m.lora_forward(dev["x"], dev["A"], dev["B"], idx, w, shape.scale, out=base.clone(), accumulate=True)
    assert util.rel_max_err(full, out.to(torch.float64).cpu().numpy()) <= 2 * util.tol(shape)


def test_dense_route_exact_ties_and_zero_gate():
    """Duplicated gate columns tie exactly: the lower index wins on this path too; a zero gate picks 0..k-1."""
    shape = LS(300, 512, 264, 12, 8, 3, 2.0, "bf16")
    ops, dev = util.make_case(shape, seed=47, condition=False)
    Wg = ops["W_gate"].copy()
    Wg[:, 5] = Wg[:, 2]
    Wg[:, 9] = Wg[:, 2]
    for gate in (Wg, np.zeros_like(Wg)):
        g = torch.from_numpy(gate).cuda()
        _, idx, w = m.linear_forward(dev["x"], dev["W"], g, None, dev["A"], dev["B"], 3, 2.0, return_routing=True)
        idx = _np(idx)
        if not gate.any():
            assert np.array_equal(idx, np.tile(np.arange(3, dtype=np.int32), (300, 1)))
            np.testing.assert_allclose(_np(w), 1.0 / 3, rtol=0, atol=1e-7)
        else:
            has2 = (idx == 2).any(axis=1)
            # whenever one of the tied columns is chosen, the lowest of them (2) is among the choices
            assert np.all(has2 | ~((idx == 5) | (idx == 9)).any(axis=1))
            assert np.all(~(idx == 9).any(axis=1) | (idx == 5).any(axis=1))


GRAPH_SHAPES = [
    LS(33, 1024, 520, 28, 8, 2, 2.0, "bf16", "uniform", "graph-decode"),
    LS(333, 1024, 520, 28, 8, 2, 2.0, "bf16", "zipf", "graph-dense-route"),
    LS(400, 1024, 520, 28, 16, 2, 2.0, "bf16", "uniform", "graph-bucketed"),
    # dense routing in front of the fused GEMM (too many output tiles for the split-K form)
    LS(2500, 512, 2056, 28, 8, 2, 2.0, "bf16", "uniform", "graph-dense-route-fused-gemm"),
]


@pytest.mark.parametrize("shape", GRAPH_SHAPES, ids=lambda s: s.name)
def test_layer_call_replays_from_a_hip_graph(shape):
    """The library allocates nothing and records no memset: a captured call replays bit-identically on new inputs."""
    ops, dev = util.make_case(shape, seed=48, condition=False)
    dt = util.torch_dtype(shape)
    packed = m.pack_weights(dev["W_gate"], dev["A"], dev["B"])
    ws = torch.empty(m.workspace_bytes(shape.T, shape.d_in, shape.d_out, shape.N, shape.r, shape.k, dt),
                     dtype=torch.uint8, device="cuda")
    x_in = dev["x"].clone()
    out = torch.empty((shape.T, shape.d_out), dtype=dt, device="cuda")
    args = (dev["W"], dev["W_gate"], dev["bias"], dev["A"], dev["B"], shape.k, shape.scale)
    m.linear_forward(x_in, *args, out=out, ws=ws, packed=packed)   # first call sets the kernels' LDS attributes
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            m.linear_forward(x_in, *args, out=out, ws=ws, packed=packed)
    torch.cuda.synchronize()
    gen_t = torch.Generator(device="cuda").manual_seed(5)
    for rep in range(3):
        x_new = torch.randn(dev["x"].shape, generator=gen_t, device="cuda", dtype=torch.float32).to(dt)
        ref = m.linear_forward(x_new, *args, packed=packed)           # eager, own output and workspace
        torch.cuda.synchronize()
        x_in.copy_(x_new)
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref), f"replay {rep} differs from the eager call"


@pytest.mark.parametrize("T", [40, 300, 2500, 9000])
def test_layer_call_does_not_depend_on_workspace_contents(T):
    """The workspace arrives uninitialised: whatever it holds (zeros, all ones, random bytes, the leftovers of other
    calls), the result is the same, call after call."""
    shape = LS(T, 512, 2056, 28, 8, 2, 2.0, "bf16", "zipf", "workspace-garbage")
    ops, dev = util.make_case(shape, seed=55, condition=False)
    dt = torch.bfloat16
    packed = m.pack_weights(dev["W_gate"], dev["A"], dev["B"])
    args = (dev["x"], dev["W"], dev["W_gate"], dev["bias"], dev["A"], dev["B"], shape.k, shape.scale)
    ref, idx_ref, w_ref = m.linear_forward(*args, packed=packed, return_routing=True)
    nbytes = m.workspace_bytes(shape.T, shape.d_in, shape.d_out, shape.N, shape.r, shape.k, dt)
    gen_t = torch.Generator(device="cuda").manual_seed(9)
    fills = [lambda n: torch.zeros(n, dtype=torch.uint8, device="cuda"),
             lambda n: torch.full((n,), 255, dtype=torch.uint8, device="cuda"),
             lambda n: torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda", generator=gen_t),
             lambda n: torch.full((n,), 1, dtype=torch.uint8, device="cuda")]
    for fill in fills:
        ws = fill(nbytes)
        for rep in range(2):   # the second call finds what the first one left
            out, idx, w = m.linear_forward(*args, packed=packed, ws=ws, return_routing=True)
            torch.cuda.synchronize()
            assert torch.equal(idx, idx_ref) and torch.equal(w, w_ref) and torch.equal(out, ref)


@pytest.mark.parametrize("r,N,path", [(12, 28, "bucketed"), (8, 28, "dense"), (16, 28, "rank16")],
                         ids=["bucketed-r12", "dense-r8", "r16"])
def test_many_tokens_small_layer_sampled_rows(r, N, path):
    """T = 70000: index arithmetic at scale on the sequences a large batch can take.  Rank 12 goes through the
    bucketed path (1094 bucketing chunks, whole-K shrink), rank 8 through the dense routing products (320 rows of
    Wcat: every batch size), rank 16 through whichever of the two the tile count of the products selects."""
    shape = LS(70000, 256, 264, N, r, 2, 2.0, "bf16", "zipf", f"T=70000-{path}")
    _check_layer(shape, seed=49, rows="sample")


# ------------------------------------------------------------------ layers that share x (q/k/v, gate/up)
def _group_case(T, d_in, d_outs, N, r, k, routing, seed):
    shapes = [LS(T, d_in, d, N, r, k, 2.0, "bf16", routing, f"member{g}") for g, d in enumerate(d_outs)]
    ops0, dev0 = util.make_case(shapes[0], seed, 0)
    members, all_ops = [], []
    for g, sh in enumerate(shapes):
        ops = gen.make_layer(sh, seed, g)
        ops["x"] = ops0["x"]                      # the members share the (margin-conditioned) input of member 0
        dev = {n: util.to_dev(ops[n], torch.bfloat16) for n in ("W", "A", "B")}
        dev["W_gate"] = util.to_dev(ops["W_gate"], torch.float32)
        dev["gate_bias"] = util.to_dev(ops["bias"], torch.float32)
        all_ops.append(ops)
        members.append(dev)
    # conditioning was done for member 0's gate only: drop the rows that are near-tied for any other member
    keep = np.ones(T, dtype=bool)
    for ops in all_ops[1:]:
        bad = margin.small_margin_rows(oracle.gate_logits(ops["x"], ops["W_gate"], ops["bias"]), k, 1e-3)
        keep[bad] = False
    return shapes, all_ops, members, dev0["x"], np.nonzero(keep)[0]


@pytest.mark.parametrize("T,d_in,d_outs,N,r,k,routing,packed", [
    (33, 1024, (520, 136, 136), 28, 8, 2, "uniform", True),      # q/k/v-like, two launches for the group
    (64, 4096, (1032, 1032), 12, 16, 3, "zipf", True),           # gate/up-like, r = 16, bias
    (8, 512, (256, 264, 136, 72), 28, 8, 2, "uniform", True),    # four members
    (33, 1024, (520, 136), 28, 8, 2, "uniform", False),          # not packed: member by member
    (300, 512, (256, 264), 28, 8, 2, "uniform", True),           # a few hundred tokens: three launches with 128-row tiles
    (16, 512, (264,), 28, 8, 2, "zipf", True),                   # a group of one is the single-layer call
    (128, 1024, (520, 136, 136), 28, 8, 2, "uniform", True),     # q/k/v-like at T = 128
    (200, 1024, (776, 776), 12, 16, 3, "zipf", True),            # gate/up-like, r = 16, bias, ragged token tile
    (130, 512, (256, 264, 136, 72), 28, 8, 2, "uniform", True),  # four members: eight matrices in one launch
    (300, 512, (256, 264), 28, 8, 2, "uniform", False),          # a few hundred tokens, not packed: member by member
    (2000, 512, (2048, 2048, 2048), 28, 8, 2, "uniform", True),  # too many output tiles for one launch: member by member
], ids=["qkv", "gate-up-r16", "four", "unpacked", "T=300", "one", "qkv-T128", "gate-up-T200-r16", "four-T130",
        "T=300-unpacked", "T=2000"])
def test_group_call_matches_oracle_and_single_calls(T, d_in, d_outs, N, r, k, routing, packed):
    shapes, all_ops, members, x, rows = _group_case(T, d_in, d_outs, N, r, k, routing, seed=50)
    for mb in members:
        mb["packed"] = m.pack_weights(mb["W_gate"], mb["A"], mb["B"]) if packed else None
    res = m.linear_forward_group(x, members, k, 2.0, return_routing=True)
    torch.cuda.synchronize()
    for sh, ops, mb, (out, idx, w) in zip(shapes, all_ops, members, res):
        ref = oracle.linear_forward(ops["x"], ops["W"], ops["W_gate"], ops["bias"], ops["A"], ops["B"], k, 2.0)
        assert np.array_equal(_np(idx)[rows], ref["idx"][rows]), f"{sh.name}: routing differs from the oracle"
        assert np.all(np.abs(_np(w) - ref["w"])[rows] <= util.weight_bound(ops, ref["idx"])[rows])
        y = out.to(torch.float64).cpu().numpy()
        err = float(np.abs(y[rows] - ref["y"][rows]).max() / np.abs(ref["y"][rows]).max())
        assert err <= util.tol(sh), f"{sh.name}: rel err {err:.3e}"
        single, idx1, w1 = m.linear_forward(x, mb["W"], mb["W_gate"], mb["gate_bias"], mb["A"], mb["B"], k, 2.0,
                                            return_routing=True, packed=mb["packed"])
        assert torch.equal(idx[torch.from_numpy(rows).cuda()], idx1[torch.from_numpy(rows).cuda()])
        assert util.rel_max_err(out, single.to(torch.float64).cpu().numpy()) <= 2 * util.tol(sh)


# ------------------------------------------------ temperature (App. A.6) and the top-1 strategy (App. A.1)
# one shape per launch sequence of the whole-layer call: decode (two launches), a few hundred tokens with the
# projection split along K, dense routing in front of the fused GEMM, bucketed (rank 12 is no multiple of 8), fp32
SEQUENCE_SHAPES = [
    LS(48, 1024, 520, 28, 8, 2, 2.0, "bf16", "uniform", "decode"),
    LS(200, 1024, 1096, 28, 8, 2, 2.0, "bf16", "zipf", "mid-split"),
    LS(2500, 512, 2056, 28, 8, 2, 2.0, "bf16", "uniform", "dense-route"),
    LS(700, 512, 264, 28, 12, 2, 2.0, "bf16", "zipf", "bucketed"),
    LS(90, 264, 136, 6, 8, 2, 2.0, "f32", "uniform", "fp32"),
]


@pytest.mark.parametrize("tau", [15.0, 20.0, 30.0])
@pytest.mark.parametrize("shape", SEQUENCE_SHAPES, ids=lambda s: s.name)
def test_linear_forward_with_temperature(shape, tau):
    """softmax(g / tau) over the selected logits in the whole-layer call (the reading of App. A.6; the formula is
    not printed in the paper): same adapters, weights and output as the oracle's with the same temperature."""
    _check_layer(shape, seed=51, inv_temperature=1.0 / tau)


@pytest.mark.parametrize("shape", SEQUENCE_SHAPES, ids=lambda s: s.name)
def test_linear_forward_top1(shape):
    """k = 1 (App. A.1): the weight is exactly 1 on every path, whatever the temperature, and the layer is
    x W + s (x A_a) B_a for the single best adapter a."""
    import dataclasses
    sh = dataclasses.replace(shape, k=1)
    _check_layer(sh, seed=52)
    ops, dev = util.make_case(sh, seed=52)
    y1, idx1, w1 = m.linear_forward(dev["x"], dev["W"], dev["W_gate"], dev["bias"], dev["A"], dev["B"], 1, sh.scale,
                                    return_routing=True)
    y2, idx2, w2 = m.linear_forward(dev["x"], dev["W"], dev["W_gate"], dev["bias"], dev["A"], dev["B"], 1, sh.scale,
                                    return_routing=True, inv_temperature=1.0 / 20.0)
    assert torch.equal(w1, torch.ones_like(w1)) and torch.equal(w2, w1)
    assert torch.equal(idx1, idx2) and torch.equal(y1, y2)


def test_group_call_with_temperature():
    """The grouped call passes the temperature on to every member (decode-sized group, two launches)."""
    shapes, all_ops, members, x, rows = _group_case(33, 1024, (520, 136), 28, 8, 2, "uniform", seed=53)
    for mb in members:
        mb["packed"] = m.pack_weights(mb["W_gate"], mb["A"], mb["B"])
    res = m.linear_forward_group(x, members, 2, 2.0, return_routing=True, inv_temperature=1.0 / 15.0)
    torch.cuda.synchronize()
    for sh, ops, (out, idx, w) in zip(shapes, all_ops, res):
        ref = oracle.linear_forward(ops["x"], ops["W"], ops["W_gate"], ops["bias"], ops["A"], ops["B"], 2, 2.0,
                                    temperature=15.0)
        assert np.array_equal(_np(idx)[rows], ref["idx"][rows])
        assert np.all(np.abs(_np(w) - ref["w"])[rows] <= util.weight_bound(ops, ref["idx"], 1.0 / 15.0)[rows])
        y = out.to(torch.float64).cpu().numpy()
        assert float(np.abs(y[rows] - ref["y"][rows]).max() / np.abs(ref["y"][rows]).max()) <= util.tol(sh)


def test_init_then_first_call_inside_a_graph_capture():
    """meteora_init sets every kernel's LDS limit ahead of time, so a call can be captured without an eager call
    of the same kind before it (this process may have launched these kernels already; the call order is what a
    capturing caller uses)."""
    m.init()
    m.init(0)
    shape = LS(130, 1024, 520, 28, 8, 2, 2.0, "bf16", "uniform", "graph-after-init")
    ops, dev = util.make_case(shape, seed=54, condition=False)
    packed = m.pack_weights(dev["W_gate"], dev["A"], dev["B"])
    ws = torch.empty(m.workspace_bytes(shape.T, shape.d_in, shape.d_out, shape.N, shape.r, shape.k, torch.bfloat16),
                     dtype=torch.uint8, device="cuda")
    out = torch.empty((shape.T, shape.d_out), dtype=torch.bfloat16, device="cuda")
    args = (dev["x"], dev["W"], dev["W_gate"], dev["bias"], dev["A"], dev["B"], shape.k, shape.scale)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            m.linear_forward(*args, out=out, ws=ws, packed=packed)
    torch.cuda.synchronize()
    ref = m.linear_forward(*args, packed=packed)
    for _ in range(2):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref)


def test_linear_forward_single_adapter_is_merged_gemm():
    """N=1,k=1: the layer is x(W + s*A*B) (Eq. 1)."""
    shape = LS(100, 256, 264, 1, 8, 1, 2.0, "f32")
    ops, dev = util.make_case(shape, seed=43, condition=False)
    y = m.linear_forward(dev["x"], dev["W"], dev["W_gate"], None, dev["A"], dev["B"], 1, 2.0)
    merged = ops["W"].astype(np.float64).T + 2.0 * ops["A"][0].astype(np.float64) @ ops["B"][0].astype(np.float64)
    assert util.rel_max_err(y, ops["x"].astype(np.float64) @ merged) <= 1e-5


# --------------------------------------------------- the seeded configurations at their full sizes
def test_config1_tiny_fp32_all_rows():
    seed, layers = gen.config_layers(1)
    _check_layer(layers[0], seed)


def test_config2_q_proj_prefill_sampled_rows():
    seed, layers = gen.config_layers(2)
    _check_layer(layers[0], seed, rows="sample")


def test_config4_decode_all_rows():
    seed, layers = gen.config_layers(4)
    for li, shape in enumerate(layers):
        _check_layer(shape, seed, li)


@pytest.mark.parametrize("li", [0, 1, 2])
def test_config3_mlp_zipf_sampled_rows(li):
    seed, layers = gen.config_layers(3)
    _check_layer(layers[li], seed, li, rows="sample")


@pytest.mark.parametrize("li", [0, 1, 2, 3, 4, 5, 6])
def test_config5_block_sampled_rows(li):
    seed, layers = gen.config_layers(5)
    _check_layer(layers[li], seed, li, rows="sample")
