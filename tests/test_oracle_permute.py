"""Pins of the oracle's permutation (stable counting sort of (token, slot) pairs by expert)."""
import numpy as np
import pytest

from oracle import oracle as O


def random_ids(g, T, E, k):
    return np.stack([g.permutation(E)[:k] for _ in range(T)]).astype(np.int32)


@pytest.mark.parametrize("T,E,k", [(1, 1, 1), (7, 3, 2), (50, 8, 2), (33, 16, 5), (64, 128, 8)])
def test_permutation_invariants_and_bruteforce(T, E, k):
    g = np.random.default_rng(T * 131 + E)
    ids = random_ids(g, T, E, k)
    X = g.standard_normal((T, 6)).astype(np.float32)
    counts, offsets, rop, por, Xp = O.permute(X, ids, E)
    R = T * k
    flat = ids.ravel()
    # dropless: every pair is kept
    assert counts.sum() == R
    np.testing.assert_array_equal(counts, np.bincount(flat, minlength=E))
    np.testing.assert_array_equal(offsets, np.concatenate([[0], np.cumsum(counts)]))
    # bijection and inverse
    assert sorted(rop.tolist()) == list(range(R))
    np.testing.assert_array_equal(por[rop], np.arange(R))
    # rows grouped by expert, stable inside a group
    e_of_row = flat[por]
    assert (np.diff(e_of_row) >= 0).all()
    for e in range(E):
        seg = por[offsets[e]:offsets[e + 1]]
        assert (np.diff(seg) > 0).all()
    # library stable sort gives the same order
    np.testing.assert_array_equal(por, np.argsort(flat, kind="stable"))
    # brute force O(R^2) definition of the rank
    for p in range(R):
        rank = sum(1 for q in range(R) if flat[q] < flat[p] or (flat[q] == flat[p] and q < p))
        assert rop[p] == rank
    # rows are bitwise copies
    np.testing.assert_array_equal(Xp, X[por // k])


def test_empty_experts_have_empty_ranges():
    ids = np.array([[0, 3], [3, 0], [0, 3]], np.int32)
    X = np.arange(6, dtype=np.float64).reshape(3, 2)
    counts, offsets, rop, por, Xp = O.permute(X, ids, 5)
    np.testing.assert_array_equal(counts, [3, 0, 0, 3, 0])
    np.testing.assert_array_equal(offsets, [0, 3, 3, 3, 6, 6])


@pytest.mark.parametrize("k", [1, 2, 4])
def test_permute_then_unpermute_is_identity(k):
    g = np.random.default_rng(k)
    T, E, d = 40, 6, 10
    ids = random_ids(g, T, E, k)
    X = g.standard_normal((T, d))
    _, _, rop, _, Xp = O.permute(X, ids, E)
    w = np.full((T, k), 1.0 / k)
    Y = O.unpermute_combine(Xp, rop, w, T)
    if k == 1:
        np.testing.assert_array_equal(Y, X)
    else:
        np.testing.assert_allclose(Y, X, rtol=1e-15, atol=0)
    # unit weights: the backward of the permutation sums the k copies
    Y1 = O.unpermute_combine(Xp, rop, None, T)
    np.testing.assert_allclose(Y1, k * X, rtol=1e-15)
