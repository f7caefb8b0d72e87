"""numpy front end of the CPU oracle (``moe_oracle.cpp``).

TEST INFRASTRUCTURE ONLY.  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this module; it imports nothing
from the HIP package.  Every function is argument marshalling around one C
entry point; the element type (fp32 or fp64 instantiation) follows the dtype of
the first floating-point argument.

Stages follow the paper's Preliminary section (mixture ``y = sum_i g_i f_i(x)``
with ``g = Softmax(TopK(x W_g))``) and the SwiGLU expert of section 3.1.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (AVX2 baseline so the binary runs on any host)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O3", "-march=x86-64-v3", "-fopenmp", "-std=c++17", "-shared", "-fPIC",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _sfx(a: np.ndarray) -> str:
    if a.dtype == np.float32:
        return "f32"
    if a.dtype == np.float64:
        return "f64"
    raise TypeError(f"oracle takes float32 or float64 arrays, got {a.dtype}")


def _p(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.c_void_p(0)
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def _i(*v):
    return [ctypes.c_int(int(x)) for x in v]


def gate_topk(X, Wg, bias, k):
    """-> ids [T,k] int32, w [T,k], logits [T,E] float64 (always fp64 accumulated)."""
    dt = X.dtype
    X, Wg = _c(X, dt), _c(Wg, dt)
    b = None if bias is None else _c(bias, dt)
    T, d = X.shape
    E = Wg.shape[1]
    ids = np.empty((T, k), np.int32)
    w = np.empty((T, k), dt)
    logits = np.empty((T, E), np.float64)
    getattr(lib(), "oracle_gate_topk_" + _sfx(X))(*_i(T, d, E, k), _p(X), _p(Wg), _p(b), _p(ids),
                                                   _p(w), _p(logits))
    return ids, w, logits


def permute(X, ids, E):
    """-> counts [E], offsets [E+1], row_of_pair [T*k], pair_of_row [T*k], Xp [T*k,d]."""
    dt = X.dtype
    X = _c(X, dt)
    ids = _c(ids, np.int32)
    T, d = X.shape
    k = ids.shape[1]
    counts = np.empty(E, np.int32)
    offsets = np.empty(E + 1, np.int32)
    rop = np.empty(T * k, np.int32)
    por = np.empty(T * k, np.int32)
    Xp = np.empty((T * k, d), dt)
    getattr(lib(), "oracle_permute_" + _sfx(X))(*_i(T, d, E, k), _p(X), _p(ids), _p(counts),
                                                 _p(offsets), _p(rop), _p(por), _p(Xp))
    return counts, offsets, rop, por, Xp


def ffn_fwd(Xp, offsets, W1, W3, W2):
    """-> Yp [R,d], A [R,f], B [R,f], H [R,f]."""
    dt = Xp.dtype
    Xp, W1, W3, W2 = _c(Xp, dt), _c(W1, dt), _c(W3, dt), _c(W2, dt)
    offsets = _c(offsets, np.int32)
    R, d = Xp.shape
    E, _, f = W1.shape
    assert W3.shape == (E, d, f) and W2.shape == (E, f, d) and offsets.shape == (E + 1,)
    assert offsets[0] == 0 and offsets[E] == R
    Yp = np.empty((R, d), dt)
    A = np.empty((R, f), dt)
    B = np.empty((R, f), dt)
    H = np.empty((R, f), dt)
    getattr(lib(), "oracle_ffn_fwd_" + _sfx(Xp))(*_i(R, d, f, E), _p(Xp), _p(offsets), _p(W1),
                                                  _p(W3), _p(W2), _p(Yp), _p(A), _p(B), _p(H))
    return Yp, A, B, H


def unpermute_combine(Yp, row_of_pair, w, T):
    """-> Y [T,d];  w None means unit weights (the backward of the permutation)."""
    dt = Yp.dtype
    Yp = _c(Yp, dt)
    rop = _c(row_of_pair, np.int32)
    d = Yp.shape[1]
    k = rop.size // T
    ww = None if w is None else _c(w, dt)
    Y = np.empty((T, d), dt)
    getattr(lib(), "oracle_unpermute_combine_" + _sfx(Yp))(*_i(T, d, k), _p(Yp), _p(rop), _p(ww),
                                                            _p(Y))
    return Y


def combine_bwd(dY, Yp, row_of_pair, w):
    """-> dYp [R,d], dw [T,k]."""
    dt = dY.dtype
    dY, Yp, w = _c(dY, dt), _c(Yp, dt), _c(w, dt)
    rop = _c(row_of_pair, np.int32)
    T, d = dY.shape
    k = w.shape[1]
    dYp = np.empty((T * k, d), dt)
    dw = np.empty((T, k), dt)
    getattr(lib(), "oracle_combine_bwd_" + _sfx(dY))(*_i(T, d, k), _p(dY), _p(Yp), _p(rop), _p(w),
                                                      _p(dYp), _p(dw))
    return dYp, dw


def ffn_bwd(Xp, offsets, W1, W3, W2, dYp):
    """-> dXp [R,d], dW1 [E,d,f], dW3 [E,d,f], dW2 [E,f,d]."""
    dt = Xp.dtype
    Xp, W1, W3, W2, dYp = _c(Xp, dt), _c(W1, dt), _c(W3, dt), _c(W2, dt), _c(dYp, dt)
    offsets = _c(offsets, np.int32)
    R, d = Xp.shape
    E, _, f = W1.shape
    assert offsets[0] == 0 and offsets[E] == R
    dXp = np.empty((R, d), dt)
    dW1 = np.empty((E, d, f), dt)
    dW3 = np.empty((E, d, f), dt)
    dW2 = np.empty((E, f, d), dt)
    getattr(lib(), "oracle_ffn_bwd_" + _sfx(Xp))(*_i(R, d, f, E), _p(Xp), _p(offsets), _p(W1),
                                                  _p(W3), _p(W2), _p(dYp), _p(dXp), _p(dW1),
                                                  _p(dW3), _p(dW2))
    return dXp, dW1, dW3, dW2


def gate_bwd(X, Wg, ids, w, dw, dX_accum=None):
    """-> dX (dX_accum + gate part, or None), dWg [d,E], dlogits [T,E]."""
    dt = X.dtype
    X, Wg, w, dw = _c(X, dt), _c(Wg, dt), _c(w, dt), _c(dw, dt)
    ids = _c(ids, np.int32)
    T, d = X.shape
    E = Wg.shape[1]
    k = ids.shape[1]
    dX = None if dX_accum is None else np.array(dX_accum, dtype=dt, order="C", copy=True)
    dWg = np.empty((d, E), dt)
    dL = np.empty((T, E), dt)
    getattr(lib(), "oracle_gate_bwd_" + _sfx(X))(*_i(T, d, E, k), _p(X), _p(Wg), _p(ids), _p(w),
                                                  _p(dw), _p(dX), _p(dWg), _p(dL))
    return dX, dWg, dL


def dense_layer_fwd(X, Wg, bias, W1, W3, W2, k):
    """The mixture written out densely -> Y [T,d], gate vector g [T,E]."""
    dt = X.dtype
    X, Wg, W1, W3, W2 = _c(X, dt), _c(Wg, dt), _c(W1, dt), _c(W3, dt), _c(W2, dt)
    b = None if bias is None else _c(bias, dt)
    T, d = X.shape
    E, _, f = W1.shape
    Y = np.empty((T, d), dt)
    g = np.empty((T, E), dt)
    getattr(lib(), "oracle_dense_layer_fwd_" + _sfx(X))(*_i(T, d, f, E, k), _p(X), _p(Wg), _p(b),
                                                         _p(W1), _p(W3), _p(W2), _p(Y), _p(g))
    return Y, g


# ---- the staged layer, chained (same intermediate tensors as the C-ABI stages)

def layer_fwd(X, Wg, bias, W1, W3, W2, k):
    E = Wg.shape[1]
    ids, w, logits = gate_topk(X, Wg, bias, k)
    counts, offsets, rop, por, Xp = permute(X, ids, E)
    Yp, A, B, H = ffn_fwd(Xp, offsets, W1, W3, W2)
    Y = unpermute_combine(Yp, rop, w, X.shape[0])
    return dict(ids=ids, w=w, logits=logits, counts=counts, offsets=offsets, row_of_pair=rop,
                pair_of_row=por, Xp=Xp, Yp=Yp, A=A, B=B, H=H, Y=Y)


def layer_bwd(X, Wg, W1, W3, W2, fwd, dY):
    """Exact derivative of layer_fwd (ids constant) -> dX, dW1, dW3, dW2, dWg + stages."""
    T = X.shape[0]
    dYp, dw = combine_bwd(dY, fwd["Yp"], fwd["row_of_pair"], fwd["w"])
    dXp, dW1, dW3, dW2 = ffn_bwd(fwd["Xp"], fwd["offsets"], W1, W3, W2, dYp)
    dX_perm = unpermute_combine(dXp, fwd["row_of_pair"], None, T)
    dX, dWg, dL = gate_bwd(X, Wg, fwd["ids"], fwd["w"], dw, dX_perm)
    return dict(dYp=dYp, dw=dw, dXp=dXp, dW1=dW1, dW3=dW3, dW2=dW2, dX_perm=dX_perm, dX=dX,
                dWg=dWg, dlogits=dL)
