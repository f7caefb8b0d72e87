"""moe_permute_static (the entry point that allocates nothing) against moe_permute, through the C ABI.

Two calls in a row on one GPU, the second with a smaller input: the static scratch array keeps the first
call's contents, so the second call must not depend on them.  Integer outputs and copied rows are compared
bit for bit with moe_permute (which the other GPU tests compare with the oracle) and with the oracle itself.
"""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2602_11686_amd import binding as B

pytestmark = pytest.mark.gpu


def random_topk(rng, T, k, E):
    """k distinct experts per token, skewed towards the low indices"""
    p = 1.0 / np.arange(1, E + 1) ** 1.2
    p /= p.sum()
    ids = np.empty((T, k), np.int32)
    for t in range(T):
        ids[t] = rng.choice(E, size=k, replace=False, p=p)
    return ids


def run_both(T, d, E, k, dtype, seed):
    rng = np.random.default_rng(seed)
    ids = random_topk(rng, T, k, E)
    x = rng.standard_normal((T, d)).astype(np.float32)
    s = B.Shape(T, d, 8, E, k, dtype)
    gx = torch.from_numpy(x).cuda().to(dtype)
    gids = torch.from_numpy(ids).cuda()
    outs = []
    for static in (False, True):
        counts = torch.full((E,), -7, dtype=torch.int32, device="cuda")
        offsets = torch.full((E + 1,), -7, dtype=torch.int32, device="cuda")
        rop = torch.full((T * k,), -7, dtype=torch.int32, device="cuda")
        por = torch.full((T * k,), -7, dtype=torch.int32, device="cuda")
        xp = torch.full((T * k, d), float("nan"), dtype=dtype, device="cuda")
        if static:
            B.moe_permute_static(s, gx, gids, counts, offsets, rop, por, xp)
        else:
            ws = torch.empty(B.moe_workspace_bytes(s), dtype=torch.uint8, device="cuda")
            B.moe_permute(s, gx, gids, counts, offsets, rop, por, xp, ws)
        torch.cuda.synchronize()
        outs.append((counts, offsets, rop, por, xp))
    for a, b in zip(*outs):
        assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                           b.view(torch.int16) if b.dtype == torch.bfloat16 else b)
    rc, ro, rrop, rpor, _ = O.permute(np.zeros((T, 1), np.float32), ids, E)
    counts, offsets, rop, por, xp = outs[1]
    np.testing.assert_array_equal(counts.cpu().numpy(), rc)
    np.testing.assert_array_equal(offsets.cpu().numpy(), ro)
    np.testing.assert_array_equal(rop.cpu().numpy(), rrop)
    np.testing.assert_array_equal(por.cpu().numpy(), rpor)
    src = torch.from_numpy(rpor // k).cuda().long()
    assert torch.equal(xp.view(torch.int16) if dtype == torch.bfloat16 else xp,
                       gx[src].view(torch.int16) if dtype == torch.bfloat16 else gx[src])


def test_two_calls_in_a_row_the_second_smaller():
    print("[no-alloc] call 1: T=4096 k=4 E=64 bf16", flush=True)
    run_both(4096, 256, 64, 4, torch.bfloat16, seed=11)
    print("[no-alloc] call 2: T=333 k=2 E=6 f32", flush=True)
    run_both(333, 64, 6, 2, torch.float32, seed=12)
    print("[no-alloc] call 3: T=1 k=1 E=2", flush=True)
    run_both(1, 8, 2, 1, torch.float32, seed=13)


def test_sizes_beyond_the_static_scratch_are_rejected():
    limit = B.moe_permute_static_max_hist_entries()
    assert limit == 65536
    # 2^22 pairs -> 512 chunks of 8192; x 256 experts = 131072 entries > limit: rejected on the host, nothing launched
    T, k, E = 1 << 20, 4, 256
    s = B.Shape(T, 8, 8, E, k, torch.float32)
    z = lambda *sh: torch.zeros(sh, dtype=torch.int32, device="cuda")
    with pytest.raises(B.MoeError, match="static scratch"):
        B.moe_permute_static(s, None, z(T, k), z(E), z(E + 1), z(T * k), z(T * k), None)
    # the largest shape that fits: 256 chunks x 256 experts
    T2 = (1 << 21) // 8
    s2 = B.Shape(T2, 8, 8, E, 8, torch.float32)
    rng = np.random.default_rng(5)
    ids = (rng.integers(0, E, size=(T2, 1)) + np.arange(8)[None, :] * 31) % E
    gids = torch.from_numpy(ids.astype(np.int32)).cuda()
    counts, offsets, rop, por = z(E), z(E + 1), z(T2 * 8), z(T2 * 8)
    B.moe_permute_static(s2, None, gids, counts, offsets, rop, por, None)
    torch.cuda.synchronize()
    rc, ro, rrop, rpor, _ = O.permute(np.zeros((T2, 1), np.float32), ids.astype(np.int32), E)
    np.testing.assert_array_equal(counts.cpu().numpy(), rc)
    np.testing.assert_array_equal(rop.cpu().numpy(), rrop)
    np.testing.assert_array_equal(por.cpu().numpy(), rpor)
