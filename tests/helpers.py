"""Shared test helpers: tiny random problems and error metrics (no method arithmetic)."""
import numpy as np


def rel_max(got, ref):
    """max |got - ref| / max |ref|  (per-tensor relative error used for every float bar)."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    den = np.abs(ref).max()
    if den == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max() / den)


def rel_max_blocks(got, ref, blocks):
    """The same metric taken block by block: every block (an expert's gradient matrix, an expert's
    group of rows) is normalised by the largest reference magnitude inside that block, so that a
    block whose values are small next to the rest of the tensor cannot hide behind it.
    `blocks` is an iterable of index expressions into both arrays; empty blocks are skipped.
    Returns (worst error, index of the worst block)."""
    worst, where = 0.0, None
    for i, b in enumerate(blocks):
        r = np.asarray(ref[b], dtype=np.float64)
        if r.size == 0:
            continue
        e = rel_max(np.asarray(got[b], dtype=np.float64), r)
        if e > worst:
            worst, where = e, i
    return worst, where


def row_blocks(offsets):
    """One slice of rows per expert (the experts' groups of a permuted tensor)."""
    return [slice(int(offsets[e]), int(offsets[e + 1])) for e in range(len(offsets) - 1)]


def tiny_problem(seed, T=12, d=16, f=24, E=4, k=2, dtype=np.float64, wstd=0.3, bias=True):
    g = np.random.default_rng(seed)
    X = g.standard_normal((T, d)).astype(dtype)
    Wg = (g.standard_normal((d, E)) * 0.5).astype(dtype)
    b = (g.standard_normal(E) * 0.3).astype(dtype) if bias else None
    W1 = (g.standard_normal((E, d, f)) * wstd).astype(dtype)
    W3 = (g.standard_normal((E, d, f)) * wstd).astype(dtype)
    W2 = (g.standard_normal((E, f, d)) * wstd).astype(dtype)
    dY = g.standard_normal((T, d)).astype(dtype)
    return X, Wg, b, W1, W3, W2, dY
