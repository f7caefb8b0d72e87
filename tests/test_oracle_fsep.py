"""Pins of the FSEP layout oracle: closed forms of section 3.1 (communication analysis) and identities."""
import numpy as np
import pytest

from oracle import fsep_oracle as F


def hosted_from(rng, N, E, C, empty=0):
    """every expert at least once when N*C >= E, the rest random; a few empty slots"""
    slots = list(range(E)) + list(rng.integers(0, E, size=N * C - E)) if N * C >= E else list(rng.integers(0, E, size=N * C))
    slots = np.array(slots[:N * C])
    rng.shuffle(slots)
    h = slots.reshape(N, C).astype(np.int32)
    for _ in range(empty):
        h[rng.integers(N), rng.integers(C)] = -1
    return h


@pytest.mark.parametrize("seed", range(6))
def test_unshard_of_shard_restores_the_hosted_experts(seed):
    rng = np.random.default_rng(seed)
    N, E, C = int(rng.choice([2, 4, 8])), int(rng.integers(1, 9)), int(rng.integers(1, 4))
    psi = N * int(rng.integers(1, 40))
    W = rng.standard_normal((E, psi))
    h = hosted_from(rng, N, E, C, empty=1)
    R = F.unshard(F.shard(W, N), h)
    for i in range(N):
        for c in range(C):
            if h[i, c] < 0:
                assert not R[i, c].any()
            else:
                np.testing.assert_array_equal(R[i, c], W[h[i, c]])


@pytest.mark.parametrize("seed", range(6))
def test_reshard_is_the_adjoint_of_unshard(seed):
    """<unshard(S), G> == <S, reshard(G)> for all S, G: reshard routes and adds exactly what unshard copies."""
    rng = np.random.default_rng(10 + seed)
    N, E, C = int(rng.choice([2, 4])), int(rng.integers(1, 6)), int(rng.integers(1, 4))
    chunk = int(rng.integers(1, 20))
    S = rng.standard_normal((N, E, chunk))
    G = rng.standard_normal((N, C, N * chunk))
    h = hosted_from(rng, N, E, C, empty=1)
    assert np.isclose((F.unshard(S, h) * G).sum(), (S * F.reshard(G, h, E)).sum(), rtol=1e-12)


def test_reshard_sums_replicas_and_zeroes_unhosted_experts():
    N, E, C, chunk = 2, 3, 2, 2
    h = np.array([[0, 1], [0, -1]], np.int32)                 # expert 0 twice, expert 1 once, expert 2 nowhere
    G = np.arange(N * C * N * chunk, dtype=np.float64).reshape(N, C, N * chunk)
    out = F.reshard(G, h, E)
    np.testing.assert_array_equal(out[0, 0], G[0, 0, :2] + G[1, 0, :2])
    np.testing.assert_array_equal(out[1, 0], G[0, 0, 2:] + G[1, 0, 2:])
    np.testing.assert_array_equal(out[:, 1].reshape(-1), G[0, 1])
    assert not out[:, 2].any()


def test_communication_volume_closed_form():
    """V_fsep = C (P-1)/P Psi per device; against FSDP+EP the ratio (P_fsep-1) P_fsdp / (P_fsep (P_fsdp-1)) is
    about 1.1 for P_fsep = 32, P_fsdp = 8 (section 3.1, communication analysis)."""
    N, C, psi = 32, 2, 32 * 1000
    assert F.unshard_volume_per_rank(N, C, psi) == C * (N - 1) * psi // N
    # count it: values of restored[i] whose source rank differs from i
    h = np.tile(np.arange(C, dtype=np.int32), (N, 1))
    src_rank = np.repeat(np.arange(N), psi // N)
    assert int((src_rank != 5).sum()) * C == F.unshard_volume_per_rank(N, C, psi)
    v_fsdp = (8 - 1) / 8 * C * psi
    assert F.unshard_volume_per_rank(N, C, psi) / v_fsdp == pytest.approx((32 - 1) * 8 / (32 * (8 - 1)))
    assert F.unshard_volume_per_rank(N, C, psi) / v_fsdp == pytest.approx(1.107, abs=1e-3)
