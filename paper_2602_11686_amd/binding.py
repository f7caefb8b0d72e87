"""ctypes binding of libmoe.so: same names as the C ABI (include/moe.h).

Argument marshalling only: every function takes torch tensors that already live
on the GPU, checks dtype/shape/contiguity, passes ``data_ptr()`` and torch's
current stream, and raises ``MoeError`` on a non-zero status.  No arithmetic of
the layer happens in Python, and there is no CPU fallback: importing works
anywhere (so the exported symbols can be checked), but calling without the
built library or without a GPU raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe.so")

MOE_F32, MOE_BF16 = 0, 1

EXPORTS = [
    "moe_status_string", "moe_last_error", "moe_abi_version", "moe_workspace_bytes", "moe_gate_topk",
    "moe_permute", "moe_grouped_ffn_fwd", "moe_grouped_ffn_bwd", "moe_unpermute_combine", "moe_combine_bwd",
    "moe_gate_topk_bwd", "moe_permute_lite", "moe_grouped_ffn_fwd_groups", "moe_permute_static",
    "moe_permute_static_max_hist_entries", "moe_grouped_ffn_bwd_groups", "moe_grouped_ffn_fwd_products",
    "moe_grouped_ffn_bwd_products",
]
_NOT_A_STATUS = {"moe_status_string", "moe_last_error", "moe_abi_version", "moe_workspace_bytes",
                 "moe_permute_static_max_hist_entries"}


class MoeError(RuntimeError):
    pass


class _CShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("T", "d", "f", "E", "k", "dtype")]


@dataclass(frozen=True)
class Shape:
    T: int
    d: int
    f: int
    E: int
    k: int
    dtype: torch.dtype  # torch.bfloat16 or torch.float32

    @property
    def R(self) -> int:
        return self.T * self.k

    def c(self) -> _CShape:
        if self.dtype not in (torch.bfloat16, torch.float32):
            raise MoeError(f"dtype {self.dtype} is not supported (bfloat16 or float32)")
        return _CShape(self.T, self.d, self.f, self.E, self.k, MOE_BF16 if self.dtype == torch.bfloat16 else MOE_F32)


_lib = None


def lib() -> ctypes.CDLL:
    """Load libmoe.so; fails loudly if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise MoeError(f"{LIB_PATH} is missing: run `python -m paper_2602_11686_amd.build` "
                           "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        L.moe_status_string.restype = ctypes.c_char_p
        L.moe_status_string.argtypes = [ctypes.c_int]
        L.moe_last_error.restype = ctypes.c_char_p
        L.moe_workspace_bytes.restype = ctypes.c_size_t
        L.moe_workspace_bytes.argtypes = [ctypes.POINTER(_CShape)]
        L.moe_permute_static_max_hist_entries.restype = ctypes.c_size_t
        L.moe_permute_static_max_hist_entries.argtypes = []
        for name in EXPORTS:
            if name not in _NOT_A_STATUS:
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _check(status: int, who: str):
    if status != 0:
        L = lib()
        raise MoeError(f"{who}: {L.moe_status_string(status).decode()} - {L.moe_last_error().decode()}")


def _ptr(t: Optional[torch.Tensor], dtype, shape, name: str):
    if t is None:
        return ctypes.c_void_p(0)
    if not t.is_cuda:
        raise MoeError(f"{name} must be a GPU tensor")
    if t.dtype != dtype:
        raise MoeError(f"{name} has dtype {t.dtype}, expected {dtype}")
    if tuple(t.shape) != tuple(shape):
        raise MoeError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    if not t.is_contiguous():
        raise MoeError(f"{name} must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _ws(ws: torch.Tensor):
    if not ws.is_cuda or ws.dtype != torch.uint8 or not ws.is_contiguous():
        raise MoeError("workspace must be a contiguous uint8 GPU tensor")
    return ctypes.c_void_p(ws.data_ptr()), ctypes.c_size_t(ws.numel())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def moe_workspace_bytes(s: Shape) -> int:
    c = s.c()
    n = lib().moe_workspace_bytes(ctypes.byref(c))
    if n == 0:
        raise MoeError("moe_workspace_bytes: " + lib().moe_last_error().decode())
    return int(n)


def moe_gate_topk(s: Shape, x, w_gate, bias, topk_ids, topk_w, logits, ws):
    c = s.c()
    wp, wn = _ws(ws)
    _check(lib().moe_gate_topk(ctypes.byref(c), _ptr(x, s.dtype, (s.T, s.d), "x"),
                               _ptr(w_gate, s.dtype, (s.d, s.E), "w_gate"),
                               _ptr(bias, torch.float32, (s.E,), "bias"),
                               _ptr(topk_ids, torch.int32, (s.T, s.k), "topk_ids"),
                               _ptr(topk_w, torch.float32, (s.T, s.k), "topk_w"),
                               _ptr(logits, torch.float32, (s.T, s.E), "logits"), wp, wn, _stream()),
           "moe_gate_topk")


def moe_permute(s: Shape, x, topk_ids, counts, offsets, row_of_pair, pair_of_row, x_perm, ws):
    c = s.c()
    wp, wn = _ws(ws)
    _check(lib().moe_permute(ctypes.byref(c), _ptr(x, s.dtype, (s.T, s.d), "x"),
                             _ptr(topk_ids, torch.int32, (s.T, s.k), "topk_ids"),
                             _ptr(counts, torch.int32, (s.E,), "counts"),
                             _ptr(offsets, torch.int32, (s.E + 1,), "offsets"),
                             _ptr(row_of_pair, torch.int32, (s.R,), "row_of_pair"),
                             _ptr(pair_of_row, torch.int32, (s.R,), "pair_of_row"),
                             _ptr(x_perm, s.dtype, (s.R, s.d), "x_perm"), wp, wn, _stream()),
           "moe_permute")


def moe_permute_static_max_hist_entries() -> int:
    return int(lib().moe_permute_static_max_hist_entries())


def moe_permute_static(s: Shape, x, topk_ids, counts, offsets, row_of_pair, pair_of_row, x_perm):
    """moe_permute without a workspace: scratch in a static device array of the library (allocates nothing)."""
    c = s.c()
    _check(lib().moe_permute_static(ctypes.byref(c), _ptr(x, s.dtype, (s.T, s.d), "x"),
                                    _ptr(topk_ids, torch.int32, (s.T, s.k), "topk_ids"),
                                    _ptr(counts, torch.int32, (s.E,), "counts"),
                                    _ptr(offsets, torch.int32, (s.E + 1,), "offsets"),
                                    _ptr(row_of_pair, torch.int32, (s.R,), "row_of_pair"),
                                    _ptr(pair_of_row, torch.int32, (s.R,), "pair_of_row"),
                                    _ptr(x_perm, s.dtype, (s.R, s.d), "x_perm"), _stream()),
           "moe_permute_static")


def moe_grouped_ffn_fwd(s: Shape, x_perm, offsets, w1, w3, w2, y_perm, a_save, b_save, ws):
    c = s.c()
    wp, wn = _ws(ws)
    _check(lib().moe_grouped_ffn_fwd(ctypes.byref(c), _ptr(x_perm, s.dtype, (s.R, s.d), "x_perm"),
                                     _ptr(offsets, torch.int32, (s.E + 1,), "offsets"),
                                     _ptr(w1, s.dtype, (s.E, s.d, s.f), "w1"),
                                     _ptr(w3, s.dtype, (s.E, s.d, s.f), "w3"),
                                     _ptr(w2, s.dtype, (s.E, s.f, s.d), "w2"),
                                     _ptr(y_perm, s.dtype, (s.R, s.d), "y_perm"),
                                     _ptr(a_save, s.dtype, (s.R, s.f), "a_save"),
                                     _ptr(b_save, s.dtype, (s.R, s.f), "b_save"), wp, wn, _stream()),
           "moe_grouped_ffn_fwd")


def moe_permute_lite(s: Shape, G: int, x, topk_ids, rep_begin, rep_group, expert_counts, group_counts, group_offsets,
                     row_of_pair, pair_of_row, x_perm, table_errors, ws):
    c = s.c()
    wp, wn = _ws(ws)
    n_rep = int(rep_group.numel())
    _check(lib().moe_permute_lite(ctypes.byref(c), ctypes.c_int32(G), ctypes.c_int32(n_rep),
                                  _ptr(x, s.dtype, (s.T, s.d), "x"),
                                  _ptr(topk_ids, torch.int32, (s.T, s.k), "topk_ids"),
                                  _ptr(rep_begin, torch.int32, (s.E + 1,), "rep_begin"),
                                  _ptr(rep_group, torch.int32, (n_rep,), "rep_group"),
                                  _ptr(expert_counts, torch.int32, (s.E,), "expert_counts"),
                                  _ptr(group_counts, torch.int32, (G,), "group_counts"),
                                  _ptr(group_offsets, torch.int32, (G + 1,), "group_offsets"),
                                  _ptr(row_of_pair, torch.int32, (s.R,), "row_of_pair"),
                                  _ptr(pair_of_row, torch.int32, (s.R,), "pair_of_row"),
                                  _ptr(x_perm, s.dtype, (s.R, s.d), "x_perm"),
                                  _ptr(table_errors, torch.int32, (1,), "table_errors"), wp, wn, _stream()),
           "moe_permute_lite")


def moe_grouped_ffn_fwd_groups(s: Shape, G: int, expert_of_group, x_perm, group_offsets, w1, w3, w2, y_perm, a_save,
                               b_save, ws):
    c = s.c()
    wp, wn = _ws(ws)
    _check(lib().moe_grouped_ffn_fwd_groups(ctypes.byref(c), ctypes.c_int32(G),
                                            _ptr(expert_of_group, torch.int32, (G,), "expert_of_group"),
                                            _ptr(x_perm, s.dtype, (s.R, s.d), "x_perm"),
                                            _ptr(group_offsets, torch.int32, (G + 1,), "group_offsets"),
                                            _ptr(w1, s.dtype, (s.E, s.d, s.f), "w1"),
                                            _ptr(w3, s.dtype, (s.E, s.d, s.f), "w3"),
                                            _ptr(w2, s.dtype, (s.E, s.f, s.d), "w2"),
                                            _ptr(y_perm, s.dtype, (s.R, s.d), "y_perm"),
                                            _ptr(a_save, s.dtype, (s.R, s.f), "a_save"),
                                            _ptr(b_save, s.dtype, (s.R, s.f), "b_save"), wp, wn, _stream()),
           "moe_grouped_ffn_fwd_groups")


def moe_grouped_ffn_fwd_products(s: Shape, x_perm, offsets, w1, w3, w2, y_perm, h_save, p_save, q_save):
    c = s.c()
    _check(lib().moe_grouped_ffn_fwd_products(ctypes.byref(c), _ptr(x_perm, s.dtype, (s.R, s.d), "x_perm"),
                                              _ptr(offsets, torch.int32, (s.E + 1,), "offsets"),
                                              _ptr(w1, s.dtype, (s.E, s.d, s.f), "w1"),
                                              _ptr(w3, s.dtype, (s.E, s.d, s.f), "w3"),
                                              _ptr(w2, s.dtype, (s.E, s.f, s.d), "w2"),
                                              _ptr(y_perm, s.dtype, (s.R, s.d), "y_perm"),
                                              _ptr(h_save, s.dtype, (s.R, s.f), "h_save"),
                                              _ptr(p_save, s.dtype, (s.R, s.f), "p_save"),
                                              _ptr(q_save, s.dtype, (s.R, s.f), "q_save"), _stream()),
           "moe_grouped_ffn_fwd_products")


def moe_grouped_ffn_bwd_products(s: Shape, x_perm, offsets, w1, w3, w2, h_save, p_save, q_save, dy_perm, dx_perm,
                                 dw1, dw3, dw2, ws):
    c = s.c()
    wp, wn = _ws(ws)
    _check(lib().moe_grouped_ffn_bwd_products(ctypes.byref(c), _ptr(x_perm, s.dtype, (s.R, s.d), "x_perm"),
                                              _ptr(offsets, torch.int32, (s.E + 1,), "offsets"),
                                              _ptr(w1, s.dtype, (s.E, s.d, s.f), "w1"),
                                              _ptr(w3, s.dtype, (s.E, s.d, s.f), "w3"),
                                              _ptr(w2, s.dtype, (s.E, s.f, s.d), "w2"),
                                              _ptr(h_save, s.dtype, (s.R, s.f), "h_save"),
                                              _ptr(p_save, s.dtype, (s.R, s.f), "p_save"),
                                              _ptr(q_save, s.dtype, (s.R, s.f), "q_save"),
                                              _ptr(dy_perm, s.dtype, (s.R, s.d), "dy_perm"),
                                              _ptr(dx_perm, s.dtype, (s.R, s.d), "dx_perm"),
                                              _ptr(dw1, s.dtype, (s.E, s.d, s.f), "dw1"),
                                              _ptr(dw3, s.dtype, (s.E, s.d, s.f), "dw3"),
                                              _ptr(dw2, s.dtype, (s.E, s.f, s.d), "dw2"), wp, wn, _stream()),
           "moe_grouped_ffn_bwd_products")


def moe_grouped_ffn_bwd(s: Shape, x_perm, offsets, w1, w3, w2, a_save, b_save, dy_perm, dx_perm, dw1, dw3, dw2, ws):
    c = s.c()
    wp, wn = _ws(ws)
    _check(lib().moe_grouped_ffn_bwd(ctypes.byref(c), _ptr(x_perm, s.dtype, (s.R, s.d), "x_perm"),
                                     _ptr(offsets, torch.int32, (s.E + 1,), "offsets"),
                                     _ptr(w1, s.dtype, (s.E, s.d, s.f), "w1"),
                                     _ptr(w3, s.dtype, (s.E, s.d, s.f), "w3"),
                                     _ptr(w2, s.dtype, (s.E, s.f, s.d), "w2"),
                                     _ptr(a_save, s.dtype, (s.R, s.f), "a_save"),
                                     _ptr(b_save, s.dtype, (s.R, s.f), "b_save"),
                                     _ptr(dy_perm, s.dtype, (s.R, s.d), "dy_perm"),
                                     _ptr(dx_perm, s.dtype, (s.R, s.d), "dx_perm"),
                                     _ptr(dw1, s.dtype, (s.E, s.d, s.f), "dw1"),
                                     _ptr(dw3, s.dtype, (s.E, s.d, s.f), "dw3"),
                                     _ptr(dw2, s.dtype, (s.E, s.f, s.d), "dw2"), wp, wn, _stream()),
           "moe_grouped_ffn_bwd")


def moe_grouped_ffn_bwd_groups(s: Shape, G: int, expert_of_group, x_perm, group_offsets, w1, w3, w2, a_save, b_save,
                               dy_perm, dx_perm, dw1_groups, dw3_groups, dw2_groups, ws):
    c = s.c()
    wp, wn = _ws(ws)
    _check(lib().moe_grouped_ffn_bwd_groups(ctypes.byref(c), ctypes.c_int32(G),
                                            _ptr(expert_of_group, torch.int32, (G,), "expert_of_group"),
                                            _ptr(x_perm, s.dtype, (s.R, s.d), "x_perm"),
                                            _ptr(group_offsets, torch.int32, (G + 1,), "group_offsets"),
                                            _ptr(w1, s.dtype, (s.E, s.d, s.f), "w1"),
                                            _ptr(w3, s.dtype, (s.E, s.d, s.f), "w3"),
                                            _ptr(w2, s.dtype, (s.E, s.f, s.d), "w2"),
                                            _ptr(a_save, s.dtype, (s.R, s.f), "a_save"),
                                            _ptr(b_save, s.dtype, (s.R, s.f), "b_save"),
                                            _ptr(dy_perm, s.dtype, (s.R, s.d), "dy_perm"),
                                            _ptr(dx_perm, s.dtype, (s.R, s.d), "dx_perm"),
                                            _ptr(dw1_groups, s.dtype, (G, s.d, s.f), "dw1_groups"),
                                            _ptr(dw3_groups, s.dtype, (G, s.d, s.f), "dw3_groups"),
                                            _ptr(dw2_groups, s.dtype, (G, s.f, s.d), "dw2_groups"), wp, wn, _stream()),
           "moe_grouped_ffn_bwd_groups")


def moe_unpermute_combine(s: Shape, y_perm, row_of_pair, topk_w, y):
    c = s.c()
    _check(lib().moe_unpermute_combine(ctypes.byref(c), _ptr(y_perm, s.dtype, (s.R, s.d), "y_perm"),
                                       _ptr(row_of_pair, torch.int32, (s.R,), "row_of_pair"),
                                       _ptr(topk_w, torch.float32, (s.T, s.k), "topk_w"),
                                       _ptr(y, s.dtype, (s.T, s.d), "y"), _stream()),
           "moe_unpermute_combine")


def moe_combine_bwd(s: Shape, dy, y_perm, row_of_pair, topk_w, dy_perm, dtopk_w):
    c = s.c()
    _check(lib().moe_combine_bwd(ctypes.byref(c), _ptr(dy, s.dtype, (s.T, s.d), "dy"),
                                 _ptr(y_perm, s.dtype, (s.R, s.d), "y_perm"),
                                 _ptr(row_of_pair, torch.int32, (s.R,), "row_of_pair"),
                                 _ptr(topk_w, torch.float32, (s.T, s.k), "topk_w"),
                                 _ptr(dy_perm, s.dtype, (s.R, s.d), "dy_perm"),
                                 _ptr(dtopk_w, torch.float32, (s.T, s.k), "dtopk_w"), _stream()),
           "moe_combine_bwd")


def moe_gate_topk_bwd(s: Shape, x, w_gate, topk_ids, topk_w, dtopk_w, dx_inout, dw_gate, ws):
    c = s.c()
    wp, wn = _ws(ws)
    _check(lib().moe_gate_topk_bwd(ctypes.byref(c), _ptr(x, s.dtype, (s.T, s.d), "x"),
                                   _ptr(w_gate, s.dtype, (s.d, s.E), "w_gate"),
                                   _ptr(topk_ids, torch.int32, (s.T, s.k), "topk_ids"),
                                   _ptr(topk_w, torch.float32, (s.T, s.k), "topk_w"),
                                   _ptr(dtopk_w, torch.float32, (s.T, s.k), "dtopk_w"),
                                   _ptr(dx_inout, s.dtype, (s.T, s.d), "dx_inout"),
                                   _ptr(dw_gate, torch.float32, (s.d, s.E), "dw_gate"), wp, wn, _stream()),
           "moe_gate_topk_bwd")
