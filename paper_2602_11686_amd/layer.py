"""Buffers of one MoE layer and the order of the C-ABI calls (no arithmetic).

``MoeLayerBuffers`` allocates every intermediate once (torch is used for device
memory only); ``forward`` / ``backward`` enqueue the stages of the hot path in
the order of include/moe.h on torch's current stream, with no host
synchronisation in between.
"""
from __future__ import annotations

from typing import Dict, Optional

import torch

from . import binding as B


class MoeLayerBuffers:
    def __init__(self, shape: B.Shape, backward: bool = False, save_activations: bool = True,
                 want_logits: bool = False, device: str = "cuda:0", save_products: bool = False):
        """save_products: keep H, P = B*silu'(A), Q = silu(A) for the backward pass (a_save holds P, b_save Q,
        h_save H) instead of A and B: the moe_grouped_ffn_*_products pair of calls."""
        s = self.shape = shape
        dev = torch.device(device)
        i32 = dict(dtype=torch.int32, device=dev)
        f32 = dict(dtype=torch.float32, device=dev)
        el = dict(dtype=s.dtype, device=dev)
        self.ws = torch.empty(B.moe_workspace_bytes(s), dtype=torch.uint8, device=dev)
        self.topk_ids = torch.empty((s.T, s.k), **i32)
        self.topk_w = torch.empty((s.T, s.k), **f32)
        self.logits = torch.empty((s.T, s.E), **f32) if want_logits else None
        self.counts = torch.empty((s.E,), **i32)
        self.offsets = torch.empty((s.E + 1,), **i32)
        self.row_of_pair = torch.empty((s.R,), **i32)
        self.pair_of_row = torch.empty((s.R,), **i32)
        self.x_perm = torch.empty((s.R, s.d), **el)
        self.y_perm = torch.empty((s.R, s.d), **el)
        self.y = torch.empty((s.T, s.d), **el)
        self.a_save = self.b_save = self.h_save = None
        if backward and save_activations:
            self.a_save = torch.empty((s.R, s.f), **el)
            self.b_save = torch.empty((s.R, s.f), **el)
            if save_products:
                self.h_save = torch.empty((s.R, s.f), **el)
        if backward:
            self.dy_perm = torch.empty((s.R, s.d), **el)
            self.dtopk_w = torch.empty((s.T, s.k), **f32)
            self.dx_perm = torch.empty((s.R, s.d), **el)
            self.dx = torch.empty((s.T, s.d), **el)
            self.dw1 = torch.empty((s.E, s.d, s.f), **el)
            self.dw3 = torch.empty((s.E, s.d, s.f), **el)
            self.dw2 = torch.empty((s.E, s.f, s.d), **el)
            self.dw_gate = torch.empty((s.d, s.E), **f32)

    def forward(self, x, w_gate, bias, w1, w3, w2):
        s = self.shape
        B.moe_gate_topk(s, x, w_gate, bias, self.topk_ids, self.topk_w, self.logits, self.ws)
        B.moe_permute(s, x, self.topk_ids, self.counts, self.offsets, self.row_of_pair, self.pair_of_row,
                      self.x_perm, self.ws)
        self.ffn_fwd(w1, w3, w2)
        B.moe_unpermute_combine(s, self.y_perm, self.row_of_pair, self.topk_w, self.y)
        return self.y

    def ffn_fwd(self, w1, w3, w2):
        s = self.shape
        if self.h_save is not None:
            B.moe_grouped_ffn_fwd_products(s, self.x_perm, self.offsets, w1, w3, w2, self.y_perm, self.h_save,
                                           self.a_save, self.b_save)
        else:
            B.moe_grouped_ffn_fwd(s, self.x_perm, self.offsets, w1, w3, w2, self.y_perm, self.a_save, self.b_save,
                                  self.ws)

    def ffn_bwd(self, w1, w3, w2):
        s = self.shape
        if self.h_save is not None:
            B.moe_grouped_ffn_bwd_products(s, self.x_perm, self.offsets, w1, w3, w2, self.h_save, self.a_save,
                                           self.b_save, self.dy_perm, self.dx_perm, self.dw1, self.dw3, self.dw2,
                                           self.ws)
        else:
            B.moe_grouped_ffn_bwd(s, self.x_perm, self.offsets, w1, w3, w2, self.a_save, self.b_save, self.dy_perm,
                                  self.dx_perm, self.dw1, self.dw3, self.dw2, self.ws)

    def backward(self, x, w_gate, w1, w3, w2, dy):
        s = self.shape
        B.moe_combine_bwd(s, dy, self.y_perm, self.row_of_pair, self.topk_w, self.dy_perm, self.dtopk_w)
        self.ffn_bwd(w1, w3, w2)
        B.moe_unpermute_combine(s, self.dx_perm, self.row_of_pair, None, self.dx)
        B.moe_gate_topk_bwd(s, x, w_gate, self.topk_ids, self.topk_w, self.dtopk_w, self.dx, self.dw_gate, self.ws)
        return self.dx


def to_device(arr, dtype: torch.dtype, device: str = "cuda:0") -> torch.Tensor:
    """numpy array from the input generators -> GPU tensor (bf16 arrives as uint16 bit patterns)."""
    import numpy as np
    if arr.dtype == np.uint16:
        assert dtype == torch.bfloat16
        return torch.from_numpy(arr.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(arr).to(device=device, dtype=dtype)
