"""Pins of the dispatcher oracle (oracle/lite_oracle.py): it must agree with the count-level lite routing
of the planner oracle (a different formulation of the same appendix algorithm), reduce to the plain stable
permutation when nothing is replicated, and keep the invariants of a permutation."""
import random

import numpy as np
import pytest

from oracle import lite_oracle as D
from oracle import oracle as O
from oracle import planner_oracle as P


def random_case(seed):
    rng = random.Random(seed)
    Dn = rng.choice([1, 2, 4])
    N = Dn * rng.choice([1, 2, 3])
    C = rng.choice([1, 2, 3])
    E = rng.randint(2, N * C) if N * C >= 2 else 1
    T = rng.choice([1, 7, 64, 300])
    k = rng.randint(1, min(E, 4))
    nrng = np.random.default_rng(seed)
    w = 1.0 / np.arange(1, E + 1) ** 1.5
    ids = np.stack([nrng.choice(E, size=k, replace=False, p=w / w.sum()) for _ in range(T)]).astype(np.int32)
    R = [[int(nrng.integers(0, 50)) for _ in range(E)] for _ in range(N)]
    rank = rng.randrange(N)
    R[rank] = [int((ids == j).sum()) for j in range(E)]
    A = P.expert_relocation(P.replica_allocation(R, N, E, C), P.expert_loads(R), N, E, C, Dn)
    return N, E, C, Dn, T, k, ids, R, A, rank


@pytest.mark.parametrize("seed", range(30))
def test_group_counts_are_the_lite_routing_shares(seed):
    N, E, C, Dn, T, k, ids, R, A, rank = random_case(seed)
    G, eog, dog, rb, rg = D.dispatch_table(A, N, E, Dn, rank)
    assert G == N * C
    ec, gc, go, rop, por = D.permute_lite(ids.tolist(), E, G, rb, rg)
    assert ec == R[rank]
    S = P.lite_routing_rank(R[rank], A, N, E, Dn, rank)                 # S[j][k]: count-level Alg. 3
    for j in range(E):
        for dev in range(N):
            assert sum(gc[g] for g in range(G) if eog[g] == j and dog[g] == dev) == S[j][dev]


@pytest.mark.parametrize("seed", range(30))
def test_permutation_invariants(seed):
    N, E, C, Dn, T, k, ids, R, A, rank = random_case(seed)
    G, eog, dog, rb, rg = D.dispatch_table(A, N, E, Dn, rank)
    ec, gc, go, rop, por = D.permute_lite(ids.tolist(), E, G, rb, rg)
    Rr = T * k
    assert sorted(rop) == list(range(Rr)) and all(por[rop[p]] == p for p in range(Rr))
    assert go[0] == 0 and go[G] == Rr and all(go[g + 1] - go[g] == gc[g] for g in range(G))
    flat = ids.reshape(-1)
    for g in range(G):
        rows = range(go[g], go[g + 1])
        assert all(flat[por[r]] == eog[g] for r in rows)                 # a group holds one expert's rows
        assert all(por[r] < por[r + 1] for r in list(rows)[:-1])        # stable inside a group
    # rows bound for one device are contiguous and devices ascend
    devs = [dog[g] for g in range(G) for _ in range(gc[g])]
    assert devs == sorted(devs)
    # the blocks of an expert follow its stable order: replica r holds earlier pairs than replica r+1
    for j in range(E):
        last = -1
        for g in rg[rb[j]:rb[j + 1]]:
            for r in range(go[g], go[g + 1]):
                assert por[r] > last
                last = por[r]


@pytest.mark.parametrize("seed", range(8))
def test_without_replication_it_is_the_plain_permutation(seed):
    """One replica per expert, groups numbered like the experts: the result must be the stable counting sort
    of the main oracle (an independent C++ routine)."""
    rng = np.random.default_rng(seed)
    E, T, k = int(rng.integers(2, 9)), int(rng.integers(1, 200)), 2
    ids = np.stack([rng.choice(E, size=k, replace=False) for _ in range(T)]).astype(np.int32)
    rb, rg = list(range(E + 1)), list(range(E))
    ec, gc, go, rop, por = D.permute_lite(ids.tolist(), E, E, rb, rg)
    x = rng.standard_normal((T, 4)).astype(np.float32)
    counts, offsets, rop_ref, por_ref, _ = O.permute(x, ids, E)
    assert gc == counts.tolist() == ec and go == offsets.tolist()
    assert rop == rop_ref.tolist() and por == por_ref.tolist()


def test_worked_example():
    """By hand: E=2, expert 0 has replicas in groups 2 and 0 listed as [0, 2], expert 1 in group 1.
    ids (k=1): 0,1,0,0,1,0,0 -> expert 0 pairs 0,2,3,5,6 (5 of them: 3 to group 0, 2 to group 2),
    expert 1 pairs 1,4 -> group 1.  Rows: group 0 = pairs 0,2,3; group 1 = pairs 1,4; group 2 = pairs 5,6."""
    ids = [[0], [1], [0], [0], [1], [0], [0]]
    ec, gc, go, rop, por = D.permute_lite(ids, 2, 3, [0, 2, 3], [0, 2, 1])
    assert ec == [5, 2] and gc == [3, 2, 2] and go == [0, 3, 5, 7]
    assert por == [0, 2, 3, 1, 4, 5, 6] and rop == [0, 3, 1, 2, 4, 5, 6]
