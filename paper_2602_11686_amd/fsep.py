"""ctypes binding of the FSEP layout kernels in libmoe.so: same names as include/moe_fsep.h.
Argument marshalling only; tensors are GPU tensors owned by the caller."""
from __future__ import annotations

import ctypes

import torch

from .binding import MOE_BF16, MOE_F32, MoeError, _check, _ptr, _stream, lib

FSEP_EXPORTS = ["moe_fsep_shard", "moe_fsep_unshard", "moe_fsep_reshard"]


def _dt(dtype):
    if dtype == torch.bfloat16:
        return MOE_BF16
    if dtype == torch.float32:
        return MOE_F32
    raise MoeError(f"unsupported dtype {dtype}")


def moe_fsep_shard(N: int, experts: torch.Tensor, shards: torch.Tensor):
    E, psi = experts.shape
    _check(lib().moe_fsep_shard(ctypes.c_int32(N), ctypes.c_int32(E), ctypes.c_int64(psi), ctypes.c_int32(_dt(experts.dtype)),
                                _ptr(experts, experts.dtype, (E, psi), "experts"),
                                _ptr(shards, experts.dtype, (N, E, psi // N), "shards"), _stream()), "moe_fsep_shard")


def moe_fsep_unshard(shards: torch.Tensor, hosted: torch.Tensor, restored: torch.Tensor):
    N, E, chunk = shards.shape
    C = hosted.shape[1]
    _check(lib().moe_fsep_unshard(ctypes.c_int32(N), ctypes.c_int32(E), ctypes.c_int32(C), ctypes.c_int64(chunk * N),
                                  ctypes.c_int32(_dt(shards.dtype)), _ptr(shards, shards.dtype, (N, E, chunk), "shards"),
                                  _ptr(hosted, torch.int32, (N, C), "hosted"),
                                  _ptr(restored, shards.dtype, (N, C, chunk * N), "restored"), _stream()), "moe_fsep_unshard")


def moe_fsep_reshard(grads: torch.Tensor, hosted: torch.Tensor, grad_shards: torch.Tensor):
    N, C, psi = grads.shape
    E = grad_shards.shape[1]
    _check(lib().moe_fsep_reshard(ctypes.c_int32(N), ctypes.c_int32(E), ctypes.c_int32(C), ctypes.c_int64(psi),
                                  ctypes.c_int32(_dt(grads.dtype)), _ptr(grads, grads.dtype, (N, C, psi), "grads"),
                                  _ptr(hosted, torch.int32, (N, C), "hosted"),
                                  _ptr(grad_shards, grads.dtype, (N, E, psi // N), "grad_shards"), _stream()), "moe_fsep_reshard")
