"""CPU oracle of the FSEP parameter layout (paper section 3.1, executor: shard, unshard, reshard), for N ranks
whose buffers are held side by side.  TEST INFRASTRUCTURE ONLY; numpy indexing, no shared code with the HIP path.

shard    every expert's flattened parameter (psi values) is cut into N equal chunks; rank n keeps chunk n of
         every expert:                      shards[n][e][:] = experts[e][n*psi/N : (n+1)*psi/N]
unshard  rank i restores the C experts its layout names (an All-to-All in the real system: rank n sends its
         chunk of every expert that rank i hosts):
                                            restored[i][c][n*psi/N + o] = shards[n][hosted[i][c]][o]
         (a slot with hosted = -1 is empty: zeros)
reshard  the full gradients of the hosted experts are cut into N chunks, chunk n goes to rank n, which adds up
         what it receives for one expert from all ranks hosting a replica of it:
                                            grad_shards[n][e][o] = sum over (i,c) with hosted[i][c] == e
                                                                   of grads[i][c][n*psi/N + o]
         in ascending (i, c) order; an expert nobody hosts gets zeros.
"""
from __future__ import annotations

import numpy as np


def shard(experts: np.ndarray, N: int) -> np.ndarray:
    E, psi = experts.shape
    assert psi % N == 0
    return np.ascontiguousarray(experts.reshape(E, N, psi // N).transpose(1, 0, 2))


def unshard(shards: np.ndarray, hosted: np.ndarray) -> np.ndarray:
    N, E, chunk = shards.shape
    _, C = hosted.shape
    out = np.zeros((N, C, N * chunk), shards.dtype)
    for i in range(N):
        for c in range(C):
            e = int(hosted[i, c])
            if e < 0:
                continue
            for n in range(N):
                out[i, c, n * chunk:(n + 1) * chunk] = shards[n, e]
    return out


def reshard(grads: np.ndarray, hosted: np.ndarray, E: int) -> np.ndarray:
    """Sums in fp64 when given fp64 input (the caller rounds); ascending (rank, slot) order."""
    N, C, psi = grads.shape
    chunk = psi // N
    out = np.zeros((N, E, chunk), grads.dtype)
    for i in range(N):
        for c in range(C):
            e = int(hosted[i, c])
            if e < 0:
                continue
            for n in range(N):
                out[n, e] += grads[i, c, n * chunk:(n + 1) * chunk]
    return out


def unshard_volume_per_rank(N: int, C: int, psi: int) -> int:
    """Values a rank receives from other ranks in one unshard: C experts, all chunks but its own."""
    return C * (N - 1) * (psi // N)
