"""GPU parity of the FSEP layout kernels (include/moe_fsep.h) against oracle/fsep_oracle.py: copies are
bitwise, the gradient reduction is within one bf16 rounding of the fp64 sum (exact in fp32 for one replica)."""
import numpy as np
import pytest
import torch

from oracle import fsep_oracle as FO
from paper_2602_11686_amd import binding as B
from paper_2602_11686_amd import fsep as F
from paper_2602_11686_amd import inputs as I
from tests.gpu_common import host
from tests.helpers import rel_max

pytestmark = pytest.mark.gpu


def hosted_for(rng, N, E, C, empty):
    slots = (list(range(E)) + list(rng.integers(0, E, size=max(N * C - E, 0))))[:N * C]
    slots = np.array(slots)
    rng.shuffle(slots)
    h = slots.reshape(N, C).astype(np.int32)
    for _ in range(empty):
        h[rng.integers(N), rng.integers(C)] = -1
    return h


CASES = [  # N, E, C, psi, dtype, empty slots
    (2, 3, 2, 2 * 8 * 5, torch.bfloat16, 0),
    (4, 8, 2, 4 * 8 * 333, torch.bfloat16, 1),
    (8, 8, 2, 8 * 8 * 1031, torch.bfloat16, 2),
    (8, 5, 3, 8 * 4 * 77, torch.float32, 1),
    (32, 16, 2, 32 * 8 * 64, torch.bfloat16, 3),
    (1, 4, 4, 8 * 9, torch.bfloat16, 0),
]


@pytest.mark.parametrize("N,E,C,psi,dtype,empty", CASES)
def test_shard_unshard_reshard(N, E, C, psi, dtype, empty):
    print(f"case N={N} E={E} C={C} psi={psi} {dtype}", flush=True)
    rng = np.random.default_rng(N * 100 + E)
    if dtype == torch.bfloat16:
        Wb = I.f32_to_bf16_bits(rng.standard_normal((E, psi)).astype(np.float32))
        Gb = I.f32_to_bf16_bits(rng.standard_normal((N, C, psi)).astype(np.float32))
        W, G = I.bf16_bits_to_f32(Wb).astype(np.float64), I.bf16_bits_to_f32(Gb).astype(np.float64)
        to = lambda b: torch.tensor(b.view(np.int16), device="cuda").view(torch.bfloat16)
        Wd, Gd = to(Wb), to(Gb)
    else:
        W = rng.standard_normal((E, psi)).astype(np.float32); G = rng.standard_normal((N, C, psi)).astype(np.float32)
        Wd, Gd = torch.tensor(W, device="cuda"), torch.tensor(G, device="cuda")
        W, G = W.astype(np.float64), G.astype(np.float64)
    h = hosted_for(rng, N, E, C, empty)
    hd = torch.tensor(h, device="cuda")
    shards = torch.empty(N, E, psi // N, dtype=dtype, device="cuda")
    restored = torch.empty(N, C, psi, dtype=dtype, device="cuda")
    gsh = torch.empty(N, E, psi // N, dtype=dtype, device="cuda")
    F.moe_fsep_shard(N, Wd, shards)
    F.moe_fsep_unshard(shards, hd, restored)
    F.moe_fsep_reshard(Gd, hd, gsh)
    torch.cuda.synchronize()
    s_ref = FO.shard(W, N)
    np.testing.assert_array_equal(host(shards), s_ref)                       # copies: exact
    np.testing.assert_array_equal(host(restored), FO.unshard(s_ref, h))
    g_ref = FO.reshard(G, h, E)
    got = host(gsh)
    reps = np.array([(h == e).sum() for e in range(E)])
    for e in range(E):
        if reps[e] <= 1:
            np.testing.assert_array_equal(got[:, e], g_ref[:, e])              # one replica (or none): a copy / zeros
    tol = 2.0 ** -8 if dtype == torch.bfloat16 else 1e-6                       # one rounding of the fp32 sum
    assert np.abs(got - g_ref).max() <= tol * max(1.0, np.abs(g_ref).max())


def test_bad_arguments_are_rejected_on_the_host():
    x = torch.empty(4, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.MoeError, match="multiple"):
        F.moe_fsep_shard(3, x, torch.empty(3, 4, 21, dtype=torch.bfloat16, device="cuda"))
