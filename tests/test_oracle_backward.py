"""Pins of the oracle's backward stages: finite differences (fp64), torch autograd
of the dense definition, adjoint identities, structural zeros."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from helpers import rel_max, tiny_problem


def loss(X, Wg, b, W1, W3, W2, k, dY):
    return float((O.layer_fwd(X, Wg, b, W1, W3, W2, k)["Y"] * dY).sum())


def margins_ok(X, Wg, b, k, eps):
    """no top-k decision (membership or slot order) within eps of flipping"""
    _, _, L = O.gate_topk(X, Wg, b, k)
    s = -np.sort(-L, axis=1)
    return (np.abs(np.diff(s[:, :k + 1], axis=1)) > eps).all()


@pytest.mark.parametrize("seed,E,k", [(20, 4, 2), (21, 5, 1), (22, 6, 3)])
def test_backward_matches_central_differences(seed, E, k):
    X, Wg, b, W1, W3, W2, dY = tiny_problem(seed, T=10, d=8, f=12, E=E, k=k)
    assert margins_ok(X, Wg, b, k, 1e-3)
    fw = O.layer_fwd(X, Wg, b, W1, W3, W2, k)
    bw = O.layer_bwd(X, Wg, W1, W3, W2, fw, dY)
    g = np.random.default_rng(seed)
    h = 1e-6
    for name, arr, grad in [("X", X, bw["dX"]), ("Wg", Wg, bw["dWg"]), ("W1", W1, bw["dW1"]),
                            ("W3", W3, bw["dW3"]), ("W2", W2, bw["dW2"])]:
        flat = arr.reshape(-1)
        gflat = grad.reshape(-1)
        for idx in g.choice(flat.size, size=min(25, flat.size), replace=False):
            old = flat[idx]
            flat[idx] = old + h
            lp = loss(X, Wg, b, W1, W3, W2, k, dY)
            flat[idx] = old - h
            lm = loss(X, Wg, b, W1, W3, W2, k, dY)
            flat[idx] = old
            fd = (lp - lm) / (2 * h)
            assert abs(fd - gflat[idx]) <= 1e-6 * max(1.0, np.abs(gflat).max()), (name, idx, fd, gflat[idx])
        # a random direction: <grad, delta> equals the directional derivative
        delta = g.standard_normal(arr.shape)
        arr += h * delta
        lp = loss(X, Wg, b, W1, W3, W2, k, dY)
        arr -= 2 * h * delta
        lm = loss(X, Wg, b, W1, W3, W2, k, dY)
        arr += h * delta
        dd = (lp - lm) / (2 * h)
        assert abs(dd - (grad * delta).sum()) <= 1e-6 * max(1.0, abs(dd)), name


def torch_dense_layer(X, Wg, b, W1, W3, W2, k):
    L = X @ Wg + b
    top, idx = torch.topk(L, k, dim=1)
    g = torch.zeros_like(L).scatter(1, idx, torch.softmax(top, dim=1))
    A = torch.einsum("td,edf->etf", X, W1)
    B = torch.einsum("td,edf->etf", X, W3)
    Fx = torch.einsum("etf,efd->etd", torch.nn.functional.silu(A) * B, W2)
    return torch.einsum("te,etd->td", g, Fx), idx


@pytest.mark.parametrize("seed,E,k", [(30, 4, 2), (31, 8, 3), (32, 3, 3)])
def test_backward_matches_autograd_of_dense_definition(seed, E, k):
    X, Wg, b, W1, W3, W2, dY = tiny_problem(seed, T=14, d=10, f=18, E=E, k=k)
    assert margins_ok(X, Wg, b, min(k, E - 1), 1e-6)
    fw = O.layer_fwd(X, Wg, b, W1, W3, W2, k)
    bw = O.layer_bwd(X, Wg, W1, W3, W2, fw, dY)
    tt = [torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (X, Wg, W1, W3, W2)]
    Y, idx = torch_dense_layer(tt[0], tt[1], torch.tensor(b), tt[2], tt[3], tt[4], k)
    np.testing.assert_array_equal(idx.numpy(), fw["ids"])
    assert rel_max(fw["Y"], Y.detach().numpy()) < 1e-12
    Y.backward(torch.tensor(dY))
    for name, t in zip(("dX", "dWg", "dW1", "dW3", "dW2"), tt):
        assert rel_max(bw[name], t.grad.numpy()) < 1e-11, name


def test_fp32_oracle_agrees_with_fp64_oracle():
    X, Wg, b, W1, W3, W2, dY = tiny_problem(40, T=48, d=32, f=48, E=6, k=2)
    fw = O.layer_fwd(X, Wg, b, W1, W3, W2, 2)
    bw = O.layer_bwd(X, Wg, W1, W3, W2, fw, dY)
    c = lambda a: a.astype(np.float32)
    fw32 = O.layer_fwd(c(X), c(Wg), c(b), c(W1), c(W3), c(W2), 2)
    bw32 = O.layer_bwd(c(X), c(Wg), c(W1), c(W3), c(W2), fw32, c(dY))
    np.testing.assert_array_equal(fw32["ids"], fw["ids"])
    for n in ("Y", "Yp", "w"):
        assert rel_max(fw32[n], fw[n]) < 1e-5, n
    for n in ("dX", "dWg", "dW1", "dW3", "dW2", "dXp", "dw", "dYp"):
        assert rel_max(bw32[n], bw[n]) < 1e-4, n


def test_adjoint_identities_per_stage():
    g = np.random.default_rng(50)
    X, Wg, b, W1, W3, W2, dY = tiny_problem(50, T=12, d=10, f=14, E=4, k=2)
    fw = O.layer_fwd(X, Wg, b, W1, W3, W2, 2)
    T, R = 12, 24
    # combine is linear in Yp: <dY, C(V)> == <C^T(dY), V>
    V = g.standard_normal((R, 10))
    dYp, dw = O.combine_bwd(dY, V, fw["row_of_pair"], fw["w"])
    lhs = (dY * O.unpermute_combine(V, fw["row_of_pair"], fw["w"], T)).sum()
    assert abs(lhs - (dYp * V).sum()) < 1e-12 * abs(lhs)
    # ... and linear in w: dw is the derivative w.r.t. each weight
    assert abs((dw * fw["w"]).sum() - lhs) < 1e-12 * abs(lhs)
    # FFN is linear in W2: <dYp, F(W2 = D)> == <dW2, D>
    G = g.standard_normal((R, 10))
    D = g.standard_normal(W2.shape)
    _, _, _, dW2 = O.ffn_bwd(fw["Xp"], fw["offsets"], W1, W3, W2, G)
    YD, *_ = O.ffn_fwd(fw["Xp"], fw["offsets"], W1, W3, D)
    assert abs((G * YD).sum() - (dW2 * D).sum()) < 1e-11 * abs((G * YD).sum())
    # FFN is linear in W3 as well
    dXp, dW1, dW3, _ = O.ffn_bwd(fw["Xp"], fw["offsets"], W1, W3, W2, G)
    D3 = g.standard_normal(W3.shape)
    YD3, *_ = O.ffn_fwd(fw["Xp"], fw["offsets"], W1, D3, W2)
    assert abs((G * YD3).sum() - (dW3 * D3).sum()) < 1e-11 * abs((G * YD3).sum())


def test_softmax_backward_rows_sum_to_zero_and_scatter():
    X, Wg, b, W1, W3, W2, dY = tiny_problem(60, T=16, E=6, k=3)
    fw = O.layer_fwd(X, Wg, b, W1, W3, W2, 3)
    bw = O.layer_bwd(X, Wg, W1, W3, W2, fw, dY)
    dL = bw["dlogits"]
    np.testing.assert_allclose(dL.sum(1), 0, atol=1e-13)
    mask = np.zeros_like(dL, dtype=bool)
    np.put_along_axis(mask, fw["ids"].astype(np.int64), True, axis=1)
    assert (dL[~mask] == 0).all()
    np.testing.assert_allclose(bw["dWg"], X.T @ dL, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(bw["dX"], bw["dX_perm"] + dL @ Wg.T, rtol=1e-12, atol=1e-14)


def test_empty_experts_get_exact_zero_weight_gradients():
    X, Wg, b, W1, W3, W2, dY = tiny_problem(70, T=10, E=5, k=1)
    b = np.array([0, -1e4, 0, -1e4, 0.0])
    fw = O.layer_fwd(X, Wg, b, W1, W3, W2, 1)
    assert fw["counts"][1] == 0 and fw["counts"][3] == 0
    bw = O.layer_bwd(X, Wg, W1, W3, W2, fw, dY)
    for n in ("dW1", "dW3", "dW2"):
        assert (bw[n][1] == 0).all() and (bw[n][3] == 0).all()
        assert np.abs(bw[n][0]).max() > 0
