"""Pins of the oracle's gate (Preliminary section: g = Softmax(TopK(x W_g)))."""
import numpy as np
import pytest
from scipy.special import softmax

from oracle import oracle as O
from helpers import tiny_problem


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("k", [1, 2, 3, 5, 8])
def test_topk_matches_library_sort_and_softmax(dtype, k):
    X, Wg, b, *_ = tiny_problem(1, T=64, d=32, E=8, dtype=dtype)
    ids, w, L = O.gate_topk(X, Wg, b, k)
    # logits: textbook matmul in fp64
    Lref = X.astype(np.float64) @ Wg.astype(np.float64) + b.astype(np.float64)
    np.testing.assert_allclose(L, Lref, rtol=1e-12, atol=1e-12)
    # selection: library stable sort on (-logit) keeps the lower index on ties
    order = np.argsort(-L, axis=1, kind="stable")[:, :k]
    np.testing.assert_array_equal(ids, order)
    # weights: library softmax restricted to the selected logits
    sel = np.take_along_axis(L, order, axis=1)
    np.testing.assert_allclose(w, softmax(sel, axis=1), rtol=0, atol=2e-7 if dtype == np.float32 else 1e-14)
    # invariants
    np.testing.assert_allclose(w.sum(1), 1.0, atol=1e-6)
    assert all(len(set(r)) == k for r in ids.tolist())
    assert (np.diff(sel, axis=1) <= 0).all()
    assert ids.min() >= 0 and ids.max() < 8


def test_k_equals_E_is_full_softmax():
    X, Wg, b, *_ = tiny_problem(2, T=20, E=6)
    ids, w, L = O.gate_topk(X, Wg, b, 6)
    full = softmax(L, axis=1)
    np.testing.assert_allclose(w, np.take_along_axis(full, ids, axis=1), atol=1e-14)


def test_k1_weight_is_one():
    X, Wg, b, *_ = tiny_problem(3)
    ids, w, L = O.gate_topk(X, Wg, b, 1)
    assert (w == 1.0).all()
    np.testing.assert_array_equal(ids[:, 0], L.argmax(1))


@pytest.mark.parametrize("k", [1, 2, 4])
def test_all_equal_logits_pick_lowest_indices(k):
    X = np.zeros((5, 8))
    Wg = np.random.default_rng(0).standard_normal((8, 4))
    ids, w, L = O.gate_topk(X, Wg, None, k)
    np.testing.assert_array_equal(ids, np.tile(np.arange(k), (5, 1)))
    np.testing.assert_allclose(w, 1.0 / k, atol=1e-15)
    assert (L == 0).all()


def test_exact_tie_between_two_experts_lower_index_first():
    # experts 1 and 3 share a weight column -> identical logits for every token
    g = np.random.default_rng(5)
    X = g.standard_normal((32, 8))
    Wg = g.standard_normal((8, 4))
    Wg[:, 3] = Wg[:, 1]
    ids, w, L = O.gate_topk(X, Wg, None, 4)
    for row in ids.tolist():
        assert row.index(1) + 1 == row.index(3)  # adjacent, lower index first


def test_huge_bias_routes_everything_to_one_expert():
    X, Wg, b, *_ = tiny_problem(4, E=5)
    b = np.zeros(5)
    b[3] = 1e4
    ids, w, _ = O.gate_topk(X, Wg, b, 1)
    assert (ids == 3).all() and (w == 1).all()


def test_dense_gate_vector_is_scatter_of_topk_weights():
    X, Wg, b, W1, W3, W2, _ = tiny_problem(6, E=6, k=3)
    ids, w, _ = O.gate_topk(X, Wg, b, 3)
    _, g = O.dense_layer_fwd(X, Wg, b, W1, W3, W2, 3)
    ref = np.zeros_like(g)
    np.put_along_axis(ref, ids.astype(np.int64), w, axis=1)
    np.testing.assert_allclose(g, ref, atol=1e-15)
    assert ((g != 0).sum(1) == 3).all()
