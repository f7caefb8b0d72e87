"""Pins of the oracle's expert FFN, combine and whole-layer forward.

Expert = SwiGLU MLP without bias (section 3.1, overlap analysis); layer =
y = sum_i g_i f_i(x) (Preliminary section)."""
import json
import os

import numpy as np
import pytest
from scipy.special import expit

from oracle import oracle as O
from paper_2602_11686_amd import inputs as I
from helpers import rel_max, tiny_problem


def swiglu_np(X, W1, W3, W2):
    A = X @ W1
    return ((A * expit(A)) * (X @ W3)) @ W2


def test_single_expert_is_a_dense_swiglu_mlp():
    X, Wg, b, W1, W3, W2, _ = tiny_problem(10, T=30, d=20, f=28, E=1, k=1)
    fw = O.layer_fwd(X, Wg, b, W1, W3, W2, 1)
    assert (fw["w"] == 1).all()
    np.testing.assert_allclose(fw["Y"], swiglu_np(X, W1[0], W3[0], W2[0]), rtol=1e-12, atol=1e-13)
    # naive triple loop on a few outputs
    for (t, c) in [(0, 0), (7, 3), (29, 19)]:
        acc = 0.0
        for j in range(28):
            a = sum(X[t, i] * W1[0, i, j] for i in range(20))
            bb = sum(X[t, i] * W3[0, i, j] for i in range(20))
            acc += a / (1 + np.exp(-a)) * bb * W2[0, j, c]
        assert abs(acc - fw["Y"][t, c]) < 1e-12 * max(1, abs(acc))


@pytest.mark.parametrize("dtype,tol", [(np.float64, 1e-12), (np.float32, 2e-5)])
def test_grouped_ffn_matches_numpy_per_expert(dtype, tol):
    X, Wg, b, W1, W3, W2, _ = tiny_problem(11, T=40, d=24, f=40, E=5, k=2, dtype=dtype)
    fw = O.layer_fwd(X, Wg, b, W1, W3, W2, 2)
    off = fw["offsets"]
    for e in range(5):
        xs = fw["Xp"][off[e]:off[e + 1]].astype(np.float64)
        ref = swiglu_np(xs, W1[e].astype(np.float64), W3[e].astype(np.float64), W2[e].astype(np.float64))
        if len(xs):
            assert rel_max(fw["Yp"][off[e]:off[e + 1]], ref) < tol
    # saved activations
    np.testing.assert_allclose(fw["H"], fw["A"] * expit(fw["A"].astype(np.float64)) * fw["B"], rtol=10 * tol, atol=tol)


def test_transposed_weight_would_be_caught():
    # non-square d != f and asymmetric weights: W1[e] used as [d,f] (y = x W)
    X, Wg, b, W1, W3, W2, _ = tiny_problem(12, T=9, d=8, f=12, E=2, k=1)
    fw = O.layer_fwd(X, Wg, b, W1, W3, W2, 1)
    t = 0
    e = fw["ids"][t, 0]
    np.testing.assert_allclose(fw["Y"][t], swiglu_np(X[t:t + 1], W1[e], W3[e], W2[e])[0], rtol=1e-12)
    # swapping the roles of W1 (silu branch) and W3 changes the result
    fw2 = O.layer_fwd(X, Wg, b, W3, W1, W2, 1)
    assert rel_max(fw2["Y"], fw["Y"]) > 1e-3


@pytest.mark.parametrize("dtype,tol", [(np.float64, 1e-13), (np.float32, 1e-5)])
@pytest.mark.parametrize("E,k", [(4, 1), (4, 2), (6, 3), (8, 8)])
def test_dense_definition_equals_staged(dtype, tol, E, k):
    X, Wg, b, W1, W3, W2, _ = tiny_problem(13 + E + k, T=16, d=16, f=24, E=E, k=k, dtype=dtype)
    fw = O.layer_fwd(X, Wg, b, W1, W3, W2, k)
    Yd, _ = O.dense_layer_fwd(X, Wg, b, W1, W3, W2, k)
    assert rel_max(fw["Y"], Yd) < tol


def test_dense_definition_equals_staged_cfg1_full():
    w = I.WORKLOADS["cfg1_tiny_f32"]
    inp = I.layer_inputs(w)
    a = {n: I.widen(v) for n, v in inp.items()}
    fw = O.layer_fwd(a["x"], a["w_gate"], a["bias"], a["w1"], a["w3"], a["w2"], w.k)
    Yd, _ = O.dense_layer_fwd(a["x"], a["w_gate"], a["bias"], a["w1"], a["w3"], a["w2"], w.k)
    assert rel_max(fw["Y"], Yd) < 1e-5
    a64 = {n: v.astype(np.float64) for n, v in a.items()}
    fw64 = O.layer_fwd(a64["x"], a64["w_gate"], a64["bias"], a64["w1"], a64["w3"], a64["w2"], w.k)
    np.testing.assert_array_equal(fw["ids"], fw64["ids"])
    assert rel_max(fw["Y"], fw64["Y"]) < 1e-5


def test_identical_experts_make_routing_irrelevant():
    X, Wg, b, W1, W3, W2, _ = tiny_problem(14, T=25, d=12, f=20, E=5, k=3)
    W1[:] = W1[0]; W3[:] = W3[0]; W2[:] = W2[0]
    fw = O.layer_fwd(X, Wg, b, W1, W3, W2, 3)
    np.testing.assert_allclose(fw["Y"], swiglu_np(X, W1[0], W3[0], W2[0]), rtol=1e-11, atol=1e-13)


def test_zero_and_scaled_down_projection():
    X, Wg, b, W1, W3, W2, _ = tiny_problem(15)
    fw = O.layer_fwd(X, Wg, b, W1, W3, W2, 2)
    assert (O.layer_fwd(X, Wg, b, W1, W3, 0 * W2, 2)["Y"] == 0).all()
    np.testing.assert_allclose(O.layer_fwd(X, Wg, b, W1, W3, -2.5 * W2, 2)["Y"], -2.5 * fw["Y"], rtol=1e-13)


def test_token_permutation_equivariance():
    X, Wg, b, W1, W3, W2, _ = tiny_problem(16, T=20)
    p = np.random.default_rng(0).permutation(20)
    y = O.layer_fwd(X, Wg, b, W1, W3, W2, 2)["Y"]
    yp = O.layer_fwd(X[p], Wg, b, W1, W3, W2, 2)["Y"]
    np.testing.assert_allclose(yp, y[p], rtol=1e-13, atol=1e-15)


def test_combine_is_weighted_sum_in_slot_order():
    g = np.random.default_rng(3)
    T, k, d = 6, 3, 5
    Yp = g.standard_normal((T * k, d))
    rop = g.permutation(T * k).astype(np.int32)
    w = g.random((T, k))
    Y = O.unpermute_combine(Yp, rop, w, T)
    ref = np.einsum("tk,tkd->td", w, Yp[rop].reshape(T, k, d))
    np.testing.assert_allclose(Y, ref, rtol=1e-14)


def test_flop_closed_forms_from_the_paper():
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_closed_forms.json")) as fh:
        gold = json.load(fh)
    # 6*H*H' per routed token (three H x H' GEMMs, 2 FLOPs per multiply-add)
    for row in gold["ffn_fwd_flops"]:
        H, Hp, S, K = row["H"], row["Hprime"], row["S"], row["K"]
        assert 3 * 2 * H * Hp == row["per_token"]
        assert S * K * 6 * H * Hp == row["per_device"]
    # backward modelled as twice the forward
    assert gold["backward_over_forward"] == 2
