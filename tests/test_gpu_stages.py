"""GPU parity, stage by stage through the C ABI, against the CPU oracle (small, ragged shapes)."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2602_11686_amd import binding as B
from paper_2602_11686_amd import inputs as I
from paper_2602_11686_amd.layer import MoeLayerBuffers
from gpu_common import TOL, check_gate, dev, follow_gpu_ids, host, oracle_inputs, round_like, shape_of, tdtype
from helpers import rel_max, rel_max_blocks, row_blocks

pytestmark = pytest.mark.gpu

BASE = I.WORKLOADS["cfg2_e64k4"]
CASES = {
    # name: (T, d, f, E, k, dtype, alpha, dead)   several tiles + ragged tails + empty experts
    "bf16_ragged": dict(T=333, d=256, f=384, E=6, k=2, dtype="bf16", alpha=1.0, dead=1),
    "bf16_k4_e40": dict(T=520, d=192, f=136, E=40, k=4, dtype="bf16", alpha=0.6, dead=3),
    "bf16_one_expert": dict(T=130, d=128, f=256, E=1, k=1, dtype="bf16", alpha=0.0, dead=0),
    "bf16_k_eq_E": dict(T=70, d=64, f=72, E=3, k=3, dtype="bf16", alpha=0.5, dead=0),
    "bf16_e130": dict(T=257, d=256, f=128, E=130, k=8, dtype="bf16", alpha=0.3, dead=0),
    "bf16_e256": dict(T=400, d=256, f=64, E=256, k=8, dtype="bf16", alpha=0.2, dead=0),   # the largest expert count
    "bf16_e64_wide": dict(T=700, d=512, f=320, E=64, k=4, dtype="bf16", alpha=0.4, dead=2),
    "bf16_k6": dict(T=300, d=128, f=96, E=16, k=6, dtype="bf16", alpha=0.5, dead=1),       # k = 6 and 5: the compile-time-k
    "bf16_k5": dict(T=190, d=64, f=128, E=9, k=5, dtype="bf16", alpha=0.7, dead=0),        # and the runtime-k row kernels
    "f32_ragged": dict(T=150, d=68, f=100, E=5, k=2, dtype="f32", alpha=1.0, dead=1),
    "f32_k6": dict(T=90, d=36, f=20, E=7, k=6, dtype="f32", alpha=0.4, dead=0),
    "f32_tiny_T": dict(T=1, d=8, f=4, E=2, k=1, dtype="f32", alpha=0.0, dead=0),
}


def make(name):
    c = CASES[name]
    w = I.scaled(BASE, name=name, seed=100 + len(name), zipf_s=1.0, backward=True, target_ratio=None, **c)
    inp = I.layer_inputs(w)
    return w, inp


@pytest.fixture(scope="module", params=list(CASES))
def case(request):
    w, inp = make(request.param)
    o = oracle_inputs(inp)
    fw = O.layer_fwd(o["x"], o["w_gate"], o["bias"], o["w1"], o["w3"], o["w2"], w.k)
    bw = O.layer_bwd(o["x"], o["w_gate"], o["w1"], o["w3"], o["w2"], fw, o["dy"])
    g = {n: dev(v, w) if n != "bias" else torch.from_numpy(v).cuda() for n, v in inp.items()}
    return w, inp, o, fw, bw, g


def test_gate_topk(case):
    w, inp, o, fw, bw, g = case
    s = shape_of(w)
    buf = MoeLayerBuffers(s, want_logits=True)
    B.moe_gate_topk(s, g["x"], g["w_gate"], g["bias"], buf.topk_ids, buf.topk_w, buf.logits, buf.ws)
    torch.cuda.synchronize()
    check_gate(host(buf.topk_ids), host(buf.topk_w), host(buf.logits), fw["ids"], fw["w"], fw["logits"], w.k)
    # without the optional logits output and without bias
    ids2 = torch.empty_like(buf.topk_ids)
    w2 = torch.empty_like(buf.topk_w)
    B.moe_gate_topk(s, g["x"], g["w_gate"], g["bias"], ids2, w2, None, buf.ws)
    assert torch.equal(ids2, buf.topk_ids) and torch.equal(w2, buf.topk_w)


def test_permute_is_bit_exact(case):
    w, inp, o, fw, bw, g = case
    s = shape_of(w)
    buf = MoeLayerBuffers(s)
    ids = torch.from_numpy(fw["ids"]).cuda()
    B.moe_permute(s, g["x"], ids, buf.counts, buf.offsets, buf.row_of_pair, buf.pair_of_row, buf.x_perm, buf.ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(buf.counts), fw["counts"])
    np.testing.assert_array_equal(host(buf.offsets), fw["offsets"])
    np.testing.assert_array_equal(host(buf.row_of_pair), fw["row_of_pair"])
    np.testing.assert_array_equal(host(buf.pair_of_row), fw["pair_of_row"])
    # rows are bitwise copies of the stored tokens
    por = fw["pair_of_row"]
    assert torch.equal(buf.x_perm.cpu(), g["x"].cpu()[torch.from_numpy(por // w.k).long()])
    # indices only
    rop2 = torch.empty_like(buf.row_of_pair)
    B.moe_permute(s, None, ids, buf.counts, buf.offsets, rop2, buf.pair_of_row, None, buf.ws)
    assert torch.equal(rop2, buf.row_of_pair)


def test_grouped_ffn_fwd(case):
    w, inp, o, fw, bw, g = case
    s = shape_of(w)
    buf = MoeLayerBuffers(s, backward=True)
    xp = dev(round_like(fw["Xp"], w), w)            # exact: Xp rows are stored values
    off = torch.from_numpy(fw["offsets"]).cuda()
    B.moe_grouped_ffn_fwd(s, xp, off, g["w1"], g["w3"], g["w2"], buf.y_perm, buf.a_save, buf.b_save, buf.ws)
    torch.cuda.synchronize()
    tol = TOL[tdtype(w)]
    groups = row_blocks(fw["offsets"])
    for name, got, want in (("Yp", buf.y_perm, fw["Yp"]), ("A", buf.a_save, fw["A"]), ("B", buf.b_save, fw["B"])):
        got = host(got)
        assert rel_max(got, want) <= tol, name
        err, e = rel_max_blocks(got, want, groups)     # every expert's rows against that expert's own scale
        assert err <= tol, (name, "expert", e, err)
    # same result without saving activations
    y2 = torch.empty_like(buf.y_perm)
    B.moe_grouped_ffn_fwd(s, xp, off, g["w1"], g["w3"], g["w2"], y2, None, None, buf.ws)
    assert torch.equal(y2, buf.y_perm)


def test_unpermute_combine(case):
    w, inp, o, fw, bw, g = case
    s = shape_of(w)
    buf = MoeLayerBuffers(s)
    yp_stored = round_like(fw["Yp"], w)
    yp = dev(yp_stored, w)
    rop = torch.from_numpy(fw["row_of_pair"]).cuda()
    tw = torch.from_numpy(fw["w"].astype(np.float32)).cuda()
    B.moe_unpermute_combine(s, yp, rop, tw, buf.y)
    ref = O.unpermute_combine(I.widen(yp_stored, np.float64), fw["row_of_pair"], fw["w"].astype(np.float32).astype(np.float64), w.T)
    torch.cuda.synchronize()
    # only the final rounding separates the two
    assert rel_max(host(buf.y), ref) <= (2.0 ** -8 if w.dtype == "bf16" else 1e-6)
    B.moe_unpermute_combine(s, yp, rop, None, buf.y)
    ref1 = O.unpermute_combine(I.widen(yp_stored, np.float64), fw["row_of_pair"], None, w.T)
    assert rel_max(host(buf.y), ref1) <= (2.0 ** -8 if w.dtype == "bf16" else 1e-6)


def test_layer_forward_end_to_end(case):
    w, inp, o, fw, bw, g = case
    s = shape_of(w)
    buf = MoeLayerBuffers(s, want_logits=True)
    buf.forward(g["x"], g["w_gate"], g["bias"], g["w1"], g["w3"], g["w2"])
    torch.cuda.synchronize()
    ids_gpu = host(buf.topk_ids)
    near = check_gate(ids_gpu, host(buf.topk_w), host(buf.logits), fw["ids"], fw["w"], fw["logits"], w.k)
    fw, _, moved = follow_gpu_ids({n: v for n, v in o.items() if n != "dy"}, w, fw, ids_gpu)
    assert moved <= near                                   # only validated near-tie tokens may differ
    np.testing.assert_array_equal(host(buf.row_of_pair), fw["row_of_pair"])
    np.testing.assert_array_equal(host(buf.offsets), fw["offsets"])
    assert rel_max(host(buf.y), fw["Y"]) <= TOL[tdtype(w)]
    assert int(buf.counts.sum()) == w.T * w.k


def test_combine_bwd(case):
    w, inp, o, fw, bw, g = case
    s = shape_of(w)
    buf = MoeLayerBuffers(s, backward=True)
    yp_stored = round_like(fw["Yp"], w)
    rop = torch.from_numpy(fw["row_of_pair"]).cuda()
    tw32 = fw["w"].astype(np.float32)
    B.moe_combine_bwd(s, g["dy"], dev(yp_stored, w), rop, torch.from_numpy(tw32).cuda(), buf.dy_perm, buf.dtopk_w)
    dYp, dw = O.combine_bwd(o["dy"], I.widen(yp_stored, np.float64), fw["row_of_pair"], tw32.astype(np.float64))
    torch.cuda.synchronize()
    assert rel_max(host(buf.dy_perm), dYp) <= (2.0 ** -8 if w.dtype == "bf16" else 1e-6)
    assert rel_max(host(buf.dtopk_w), dw) <= 1e-5


def test_grouped_ffn_bwd(case):
    w, inp, o, fw, bw, g = case
    s = shape_of(w)
    buf = MoeLayerBuffers(s, backward=True)
    xp = dev(round_like(fw["Xp"], w), w)
    off = torch.from_numpy(fw["offsets"]).cuda()
    dyp_stored = round_like(bw["dYp"], w)
    ref = O.ffn_bwd(fw["Xp"], fw["offsets"], o["w1"], o["w3"], o["w2"], I.widen(dyp_stored, np.float64))
    tol = TOL[tdtype(w)]
    for saved in (True, False):
        if saved:
            B.moe_grouped_ffn_fwd(s, xp, off, g["w1"], g["w3"], g["w2"], buf.y_perm, buf.a_save, buf.b_save, buf.ws)
        a, b = (buf.a_save, buf.b_save) if saved else (None, None)
        for t in (buf.dx_perm, buf.dw1, buf.dw3, buf.dw2):
            t.fill_(float("nan"))
        B.moe_grouped_ffn_bwd(s, xp, off, g["w1"], g["w3"], g["w2"], a, b, dev(dyp_stored, w), buf.dx_perm,
                              buf.dw1, buf.dw3, buf.dw2, buf.ws)
        torch.cuda.synchronize()
        for name, got, want in (("dXp", buf.dx_perm, ref[0]), ("dW1", buf.dw1, ref[1]), ("dW3", buf.dw3, ref[2]),
                                ("dW2", buf.dw2, ref[3])):
            got = host(got)
            assert rel_max(got, want) <= tol, (name, saved)
            # every expert's block against that expert's own scale: a light expert's gradients are orders
            # of magnitude smaller than the heaviest one's and must still be right
            blocks = row_blocks(fw["offsets"]) if name == "dXp" else range(w.E)
            err, e = rel_max_blocks(got, want, blocks)
            assert err <= tol, (name, saved, "expert", e, err)
        # experts without rows: exact zeros
        for e in np.nonzero(fw["counts"] == 0)[0]:
            assert float(buf.dw1[e].abs().max()) == 0 and float(buf.dw2[e].abs().max()) == 0 \
                and float(buf.dw3[e].abs().max()) == 0


def test_grouped_ffn_products(case):
    """The pair of calls that saves H, P = B*silu'(A) and Q = silu(A): same outputs as the plain pair, the saved
    tensors against the oracle's A and B put through scipy's expit, the gradients against the oracle's."""
    from scipy.special import expit
    w, inp, o, fw, bw, g = case
    if not w.backward:
        pytest.skip("forward-only configuration")
    s = shape_of(w)
    buf = MoeLayerBuffers(s, backward=True)
    xp = dev(round_like(fw["Xp"], w), w)
    off = torch.from_numpy(fw["offsets"]).cuda()
    tol = TOL[tdtype(w)]
    h, p, q = (torch.full_like(buf.a_save, float("nan")) for _ in range(3))
    y = torch.full_like(buf.y_perm, float("nan"))
    B.moe_grouped_ffn_fwd_products(s, xp, off, g["w1"], g["w3"], g["w2"], y, h, p, q)
    B.moe_grouped_ffn_fwd(s, xp, off, g["w1"], g["w3"], g["w2"], buf.y_perm, None, None, buf.ws)
    torch.cuda.synchronize()
    assert torch.equal(y, buf.y_perm)
    A, Bm = fw["A"].astype(np.float64), fw["B"].astype(np.float64)
    sg = expit(A)
    groups = row_blocks(fw["offsets"])
    for name, got, want in (("H", h, A * sg * Bm), ("P", p, Bm * sg * (1.0 + A * (1.0 - sg))), ("Q", q, A * sg)):
        got = host(got)
        assert rel_max(got, want) <= tol, name
        err, e = rel_max_blocks(got, want, groups)
        assert err <= tol, (name, "expert", e, err)
    dyp_stored = round_like(bw["dYp"], w)
    ref = O.ffn_bwd(fw["Xp"], fw["offsets"], o["w1"], o["w3"], o["w2"], I.widen(dyp_stored, np.float64))
    for t in (buf.dx_perm, buf.dw1, buf.dw3, buf.dw2):
        t.fill_(float("nan"))
    B.moe_grouped_ffn_bwd_products(s, xp, off, g["w1"], g["w3"], g["w2"], h, p, q, dev(dyp_stored, w), buf.dx_perm,
                                   buf.dw1, buf.dw3, buf.dw2, buf.ws)
    torch.cuda.synchronize()
    for name, got, want in (("dXp", buf.dx_perm, ref[0]), ("dW1", buf.dw1, ref[1]), ("dW3", buf.dw3, ref[2]),
                            ("dW2", buf.dw2, ref[3])):
        got = host(got)
        assert rel_max(got, want) <= tol, name
        blocks = groups if name == "dXp" else range(w.E)
        err, e = rel_max_blocks(got, want, blocks)
        assert err <= tol, (name, "expert", e, err)
    for e in np.nonzero(fw["counts"] == 0)[0]:
        assert float(buf.dw1[e].abs().max()) == 0 and float(buf.dw2[e].abs().max()) == 0 \
            and float(buf.dw3[e].abs().max()) == 0


def test_gate_topk_bwd(case):
    w, inp, o, fw, bw, g = case
    s = shape_of(w)
    buf = MoeLayerBuffers(s, backward=True)
    ids = torch.from_numpy(fw["ids"]).cuda()
    tw32 = fw["w"].astype(np.float32)
    dw32 = bw["dw"].astype(np.float32)
    dx_in = round_like(bw["dX_perm"], w)
    buf.dx.copy_(dev(dx_in, w))
    B.moe_gate_topk_bwd(s, g["x"], g["w_gate"], ids, torch.from_numpy(tw32).cuda(), torch.from_numpy(dw32).cuda(),
                        buf.dx, buf.dw_gate, buf.ws)
    dX, dWg, _ = O.gate_bwd(o["x"], o["w_gate"], fw["ids"], tw32.astype(np.float64), dw32.astype(np.float64),
                            I.widen(dx_in, np.float64))
    torch.cuda.synchronize()
    assert rel_max(host(buf.dw_gate), dWg) <= 1e-4
    assert rel_max(host(buf.dx), dX) <= (2.0 ** -8 if w.dtype == "bf16" else 1e-5)


def test_layer_backward_end_to_end(case):
    w, inp, o, fw, bw, g = case
    s = shape_of(w)
    buf = MoeLayerBuffers(s, backward=True, want_logits=True)
    buf.forward(g["x"], g["w_gate"], g["bias"], g["w1"], g["w3"], g["w2"])
    buf.backward(g["x"], g["w_gate"], g["w1"], g["w3"], g["w2"], g["dy"])
    torch.cuda.synchronize()
    ids_gpu = host(buf.topk_ids)
    near = check_gate(ids_gpu, host(buf.topk_w), host(buf.logits), fw["ids"], fw["w"], fw["logits"], w.k)
    fw2, bw2, moved = follow_gpu_ids(o, w, fw, ids_gpu)    # near-tie tokens: the oracle follows the GPU's ids
    assert moved <= near
    if moved:
        fw, bw = fw2, bw2
    np.testing.assert_array_equal(host(buf.row_of_pair), fw["row_of_pair"])
    tol = TOL[tdtype(w)]
    for name, got in (("dX", buf.dx), ("dW1", buf.dw1), ("dW3", buf.dw3), ("dW2", buf.dw2), ("dWg", buf.dw_gate)):
        got = host(got)
        assert rel_max(got, bw[name]) <= tol, name
        if name in ("dW1", "dW3", "dW2"):
            err, e = rel_max_blocks(got, bw[name], range(w.E))
            assert err <= tol, (name, "expert", e, err)


def test_run_to_run_determinism(case):
    w, inp, o, fw, bw, g = case
    s = shape_of(w)
    outs = []
    for _ in range(2):
        buf = MoeLayerBuffers(s, backward=True)
        buf.forward(g["x"], g["w_gate"], g["bias"], g["w1"], g["w3"], g["w2"])
        buf.backward(g["x"], g["w_gate"], g["w1"], g["w3"], g["w2"], g["dy"])
        torch.cuda.synchronize()
        outs.append([t.clone() for t in (buf.y, buf.dx, buf.dw1, buf.dw2, buf.dw3, buf.dw_gate, buf.row_of_pair)])
    for a, b in zip(*outs):
        assert torch.equal(a, b)


# Row counts chosen around the tile edges of the grouped GEMM (one row, less than one MFMA block, one
# short of / one past a 32-row k-stage of the weight gradient, one short of / one past a 256-row tile,
# an empty expert, exactly half a tile and one past it).
EDGE_COUNTS = [1, 7, 31, 33, 255, 257, 0, 128, 129, 64, 2, 513]


# (256, 384): the MFMA-tile kernel; (192, 136): f is no multiple of 64, so the GEMMs with K = f take the plain tiled
# kernel; (64, 64): one k-stage per tile; (128, 192): two and three k-stages (the pipelined loop runs once at most);
# (320, 264): five k-stages and a last column tile 8 wide
@pytest.mark.parametrize("d,f", [(256, 384), (192, 136), (64, 64), (128, 192), (320, 264)])
def test_grouped_ffn_at_tile_edges(d, f):
    """moe_grouped_ffn_fwd / _bwd driven with a chosen count vector: every expert's rows and every expert's
    weight gradients are compared with the oracle on that expert's own scale."""
    rng = np.random.default_rng(20240 + d)
    counts = np.array(EDGE_COUNTS, np.int32)
    E, R = len(counts), int(counts.sum())
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    bits = lambda a: I.f32_to_bf16_bits(a.astype(np.float32))
    xp_b = bits(rng.standard_normal((R, d)))
    dyp_b = bits(rng.standard_normal((R, d)))
    w1_b, w3_b = bits(rng.standard_normal((E, d, f)) * 0.05), bits(rng.standard_normal((E, d, f)) * 0.05)
    w2_b = bits(rng.standard_normal((E, f, d)) * 0.05)
    wd = lambda a: I.widen(a, np.float64)
    yp, A, Bm, H = O.ffn_fwd(wd(xp_b), offsets, wd(w1_b), wd(w3_b), wd(w2_b))
    dxp, dw1, dw3, dw2 = O.ffn_bwd(wd(xp_b), offsets, wd(w1_b), wd(w3_b), wd(w2_b), wd(dyp_b))
    # T*k = R with k = 1: the shape only sizes the buffers of these two calls
    s = B.Shape(R, d, f, E, 1, torch.bfloat16)
    buf = MoeLayerBuffers(s, backward=True)
    tod = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    xp, dyp, w1, w3, w2 = tod(xp_b), tod(dyp_b), tod(w1_b), tod(w3_b), tod(w2_b)
    off = torch.from_numpy(offsets).cuda()
    groups = row_blocks(offsets)
    for saved in (True, False):
        for t in (buf.y_perm, buf.a_save, buf.b_save, buf.dx_perm, buf.dw1, buf.dw3, buf.dw2):
            t.fill_(float("nan"))
        B.moe_grouped_ffn_fwd(s, xp, off, w1, w3, w2, buf.y_perm, buf.a_save, buf.b_save, buf.ws)
        a, b = (buf.a_save, buf.b_save) if saved else (None, None)
        B.moe_grouped_ffn_bwd(s, xp, off, w1, w3, w2, a, b, dyp, buf.dx_perm, buf.dw1, buf.dw3, buf.dw2, buf.ws)
        torch.cuda.synchronize()
        for name, got, want, blocks in (("Yp", buf.y_perm, yp, groups), ("A", buf.a_save, A, groups),
                                        ("B", buf.b_save, Bm, groups), ("dXp", buf.dx_perm, dxp, groups),
                                        ("dW1", buf.dw1, dw1, range(E)), ("dW3", buf.dw3, dw3, range(E)),
                                        ("dW2", buf.dw2, dw2, range(E))):
            got = host(got)
            assert np.isfinite(got).all(), (name, saved)
            assert rel_max(got, want) <= 2e-2, (name, saved)
            err, e = rel_max_blocks(got, want, blocks)
            assert err <= 2e-2, (name, saved, "expert", e, "rows", int(counts[e]), err)
        e0 = EDGE_COUNTS.index(0)
        assert float(buf.dw1[e0].abs().max()) == 0 and float(buf.dw3[e0].abs().max()) == 0 \
            and float(buf.dw2[e0].abs().max()) == 0
    # the pair that saves products, on the same edges
    y_plain = buf.y_perm.clone()
    h = torch.full_like(buf.a_save, float("nan"))
    for t in (buf.y_perm, buf.a_save, buf.b_save, buf.dx_perm, buf.dw1, buf.dw3, buf.dw2):
        t.fill_(float("nan"))
    B.moe_grouped_ffn_fwd_products(s, xp, off, w1, w3, w2, buf.y_perm, h, buf.a_save, buf.b_save)
    B.moe_grouped_ffn_bwd_products(s, xp, off, w1, w3, w2, h, buf.a_save, buf.b_save, dyp, buf.dx_perm, buf.dw1,
                                   buf.dw3, buf.dw2, buf.ws)
    torch.cuda.synchronize()
    assert torch.equal(buf.y_perm, y_plain)
    for name, got, want, blocks in (("H", h, H, groups), ("dXp", buf.dx_perm, dxp, groups),
                                    ("dW1", buf.dw1, dw1, range(E)), ("dW3", buf.dw3, dw3, range(E)),
                                    ("dW2", buf.dw2, dw2, range(E))):
        got = host(got)
        assert np.isfinite(got).all(), name
        assert rel_max(got, want) <= 2e-2, name
        err, e = rel_max_blocks(got, want, blocks)
        assert err <= 2e-2, (name, "products", "expert", e, "rows", int(counts[e]), err)
