"""Pins of the planner oracle (oracle/planner_oracle.py) against things it did not compute itself:
hand-worked examples (tests/golden/planner_examples.json), brute force on tiny inputs, invariants of
the problem formulation (paper section 4) and closed forms."""
import itertools
import json
import os
import random

import pytest

from oracle import planner_oracle as P

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "planner_examples.json")))
COST = dict(v_comm=2.0, b_intra=8.0, b_inter=1.0, v_comp=3.0, b_comp=5.0, f_ckpt=0)


def rand_R(rng, N, E, hi=50, skew=True):
    w = [rng.random() ** (3 if skew else 0) for _ in range(E)]
    return [[int(hi * w[j] * rng.random() * 2) for j in range(E)] for _ in range(N)]


# ---------------------------------------------------------------- replica allocation (appendix Alg. 4)
def compositions(total, parts):
    if parts == 1:
        yield (total,)
        return
    for first in range(1, total - parts + 2):
        for rest in compositions(total - first, parts - 1):
            yield (first,) + rest


@pytest.mark.parametrize("seed", range(12))
def test_replica_allocation_minimises_the_heaviest_replica(seed):
    """The highest-average greedy is optimal for min max_j load_j / rep_j: brute force over every
    replica vector with the same total."""
    rng = random.Random(seed)
    N, C, E = rng.choice([(2, 2, 3), (4, 2, 4), (3, 2, 2), (4, 1, 4), (5, 1, 3)])
    R = rand_R(rng, N, E)
    rep = P.replica_allocation(R, N, E, C)
    load = P.expert_loads(R)
    assert sum(rep) == N * C and min(rep) >= 1
    best = min(max(load[j] / r[j] for j in range(E)) for r in compositions(N * C, E))
    assert max(load[j] / rep[j] for j in range(E)) == pytest.approx(best, rel=0, abs=0)


def test_replica_allocation_special_cases():
    assert P.replica_allocation([[5, 5, 5, 5]] * 4, 4, 4, 2) == [2, 2, 2, 2]          # equal loads, divisible
    assert P.replica_allocation([[0, 0, 0, 0]] * 2, 2, 4, 2) == [1, 1, 1, 1]          # N*C == E: nothing to hand out
    assert P.replica_allocation([[100, 1, 1]], 1, 3, 5) == [3, 1, 1]                   # 100/1, 100/2 > 1: both extras to expert 0
    assert P.replica_allocation([[4, 4, 0]], 1, 3, 5) == [2, 2, 1]                     # tie -> lower index first
    with pytest.raises(ValueError):
        P.replica_allocation([[1, 1, 1]], 1, 3, 2)


# ---------------------------------------------------------------- expert relocation (Alg. 1)
def test_relocation_worked_example():
    g = GOLD["relocation"]
    assert P.expert_relocation(g["expert_rep"], g["loads"], g["N"], g["E"], g["C"], g["D"]) == g["A"]


@pytest.mark.parametrize("seed", range(20))
def test_relocation_invariants(seed):
    rng = random.Random(100 + seed)
    D = rng.choice([1, 2, 4])
    N = D * rng.choice([1, 2, 3])
    C = rng.choice([1, 2, 3])
    E = rng.randint(1, N * C)
    R = rand_R(rng, N, E)
    rep = P.replica_allocation(R, N, E, C)
    A = P.expert_relocation(rep, P.expert_loads(R), N, E, C, D)
    assert [sum(A[i][j] for i in range(N)) for j in range(E)] == rep          # every replica placed
    assert all(sum(A[i]) == C for i in range(N))                               # eq. 3 as glossed: C per device
    # an expert sits twice on a device only if it has more replicas than devices, or the free slots ran out
    for j in range(E):
        if max(A[i][j] for i in range(N)) > 1:
            assert rep[j] > 1


def test_relocation_spreads_replicas_over_nodes():
    # one hot expert with 4 replicas, 4 nodes of 2 devices, plenty of room: one replica per node
    N, D, E, C = 8, 2, 5, 1
    rep, loads = [4, 1, 1, 1, 1], [400, 4, 3, 2, 1]
    A = P.expert_relocation(rep, loads, N, E, C, D)
    assert [sum(A[i][0] for i in range(n * D, n * D + D)) for n in range(4)] == [1, 1, 1, 1]
    assert all(sum(A[i]) == 1 for i in range(N))


def test_relocation_duplicates_only_when_forced():
    # 3 replicas of one expert on 2 devices: one device must take two
    A = P.expert_relocation([3, 1], [30, 1], 2, 2, 2, 2)
    assert sorted(A[i][0] for i in range(2)) == [1, 2] and sum(A[i][1] for i in range(2)) == 1


# ---------------------------------------------------------------- lite routing (appendix Alg. 3)
def test_lite_routing_worked_example():
    A = GOLD["relocation"]["A"]
    g = GOLD["lite_routing"]
    assert P.lite_routing_rank(g["R_rank"], A, 4, 4, 2, 0) == g["rank0"]
    assert P.lite_routing_rank(g["R_rank"], A, 4, 4, 2, 3) == g["rank3"]


@pytest.mark.parametrize("seed", range(20))
def test_lite_routing_invariants(seed):
    rng = random.Random(200 + seed)
    D = rng.choice([1, 2, 4])
    N = D * rng.choice([1, 2, 3])
    C = rng.choice([1, 2])
    E = rng.randint(1, N * C)
    R = rand_R(rng, N, E)
    A = P.expert_relocation(P.replica_allocation(R, N, E, C), P.expert_loads(R), N, E, C, D)
    S = P.lite_routing(R, A, N, E, D)
    for i in range(N):
        for j in range(E):
            assert sum(S[i][j]) == R[i][j]                                     # eq. 4: every token goes somewhere
            assert all(S[i][j][k] == 0 for k in range(N) if A[k][j] == 0)      # ... to a device that holds the expert
            node = range((i // D) * D, (i // D) * D + D)
            if any(A[k][j] for k in node):                                     # a replica in the node: nothing leaves it
                assert all(S[i][j][k] == 0 for k in range(N) if k not in node)
            per = [S[i][j][k] / A[k][j] for k in range(N) if A[k][j] and (S[i][j][k] or not any(A[q][j] for q in node) or k in node)]
            if per:
                assert max(per) - min(per) <= 1                                 # even split


# ---------------------------------------------------------------- cost model (section 4)
def test_time_cost_worked_example():
    g = GOLD["time_cost"]
    T, tc, tp = P.time_cost(g["S"], g["N"], g["E"], g["D"], **g["params"])
    assert (T, tc, tp) == (g["T"], g["T_comm"], g["T_comp"])


def test_time_cost_uniform_closed_form():
    # N=4 in 2 nodes, E=4, one expert per device, every device holds r tokens per expert
    N, D, E, r = 4, 2, 4, 6
    A = [[1 if i == j else 0 for j in range(E)] for i in range(N)]
    R = [[r] * E for _ in range(N)]
    S = P.lite_routing(R, A, N, E, D)
    T, tc, tp = P.time_cost(S, N, E, D, **COST)
    assert tp == 3 * COST["v_comp"] * (N * r) / COST["b_comp"]
    assert tc == pytest.approx(4 * COST["v_comm"] * N * (r / COST["b_intra"] + 2 * r / COST["b_inter"]))
    assert T == tc + tp


# ---------------------------------------------------------------- expert layout (Alg. 2)
def all_layouts(N, E, C):
    """every binary A with exactly C experts per device and every expert somewhere"""
    rows = list(itertools.combinations(range(E), C))
    for pick in itertools.product(rows, repeat=N):
        A = [[1 if j in pick[i] else 0 for j in range(E)] for i in range(N)]
        if all(any(A[i][j] for i in range(N)) for j in range(E)):
            yield A


@pytest.mark.parametrize("seed", range(6))
def test_expert_layout_against_exhaustive_search(seed):
    rng = random.Random(300 + seed)
    N, D, E, C = rng.choice([(4, 2, 2, 1), (4, 2, 3, 1), (4, 2, 4, 2), (2, 1, 3, 2)])
    R = rand_R(rng, N, E)
    A, T, idx, cands = P.expert_layout(R, N, E, C, D, eps=6, seed=seed, cost_params=COST)
    opt = min(P.time_cost(P.lite_routing(R, B, N, E, D), N, E, D, **COST)[0] for B in all_layouts(N, E, C))
    assert T >= opt - 1e-9                                   # a heuristic cannot beat the optimum under the same routing
    assert T <= 2.0 * opt + 1e-9                             # and on these sizes it stays within a factor of two
    # never worse than its own first two candidates
    for rep in cands[:2]:
        B = P.expert_relocation(rep, P.expert_loads(R), N, E, C, D)
        assert T <= P.time_cost(P.lite_routing(R, B, N, E, D), N, E, D, **COST)[0]
    assert all(sum(c) == N * C and min(c) >= 1 for c in cands) and len(cands) == 6


def test_expert_layout_is_deterministic_and_seeded():
    rng = random.Random(7)
    R = rand_R(rng, 8, 8)
    a = P.expert_layout(R, 8, 8, 2, 4, eps=8, seed=11, cost_params=COST)
    b = P.expert_layout(R, 8, 8, 2, 4, eps=8, seed=11, cost_params=COST)
    c = P.expert_layout(R, 8, 8, 2, 4, eps=8, seed=12, cost_params=COST)
    assert a == b and a[3][:2] == c[3][:2] and a[3] != c[3]


def test_splitmix64_reference_values():
    # first outputs for seed 0 of the published splitmix64 generator
    g = P.SplitMix64(0)
    assert [g.next() for _ in range(3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_rebalancing_helps_a_skewed_load():
    """The paper's motivating example (section 4, load-balancing figure): two hot experts; re-layout with
    replicas lowers the modelled time against the static one-expert-per-device layout."""
    N, D, E, C = 4, 2, 4, 2
    R = [[60, 50, 5, 5]] * N
    static = [[1, 0, 1, 0], [0, 1, 0, 1], [1, 0, 1, 0], [0, 1, 0, 1]]    # experts (0,2) / (1,3) per device pair
    t_static = P.time_cost(P.lite_routing(R, static, N, E, D), N, E, D, **COST)[0]
    _, T, _, _ = P.expert_layout(R, N, E, C, D, eps=4, seed=0, cost_params=COST)
    assert T <= t_static
