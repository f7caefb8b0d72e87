"""CPU oracle of the load-balancing planner (paper section 4: problem formulation, Alg. 1 expert
relocation, Alg. 2 expert layout, appendix Alg. 3 lite routing, appendix Alg. 4 replica allocation).

TEST INFRASTRUCTURE ONLY: plain Python loops over small lists, no vectorisation, no shared code with
the C++ planner.  Only ``tests/`` imports it.

Notation follows the paper: N devices, E experts, C expert slots per device, ``R[i][j]`` tokens on
device i routed to expert j, ``A[i][j]`` replicas of expert j restored on device i, ``S[i][j][k]``
tokens of device i for expert j that are sent to device k.  Devices ``n*D .. n*D+D-1`` form node n
(D = devices per node).

Readings taken where the paper is silent or at odds with itself (all of them are also what the C++
planner implements, so the two can be compared bit for bit):

* loads and times are IEEE doubles; an expert's per-replica load is ``load / replicas`` (one division),
  a device's load is the running sum of the per-replica loads placed on it, in placement order;
* ties: lowest expert index (replica allocation, descending sort is stable), lowest device index;
* the layout is indexed [device][expert] (the problem statement; Alg. 1's listing allocates it the other
  way round) and the per-device constraint is "C slots per device" (the gloss of eq. 3, not its formula);
* Alg. 1 may meet a replica whose least-loaded nodes have no free slot, or only devices that already
  hold the expert: nodes without an eligible device are left out before the minimum is taken, and devices
  that already hold the expert are eligible only if no other device with a free slot exists anywhere
  (keeps A binary whenever the replica count allows it, as the formulation demands);
* lite routing splits ``R[i][j]`` into ``len(replicas)`` integer shares that differ by at most one, the
  larger shares going to the lowest-indexed replicas; a device holding m replicas counts m times;
* a device sending to itself costs no communication time;
* "evenly_replicas" when N*C is not a multiple of E: floor, the remainder to the lowest-indexed experts;
* "random perturb": one replica moves from a random expert that has more than one to another random
  expert; the random numbers come from splitmix64 seeded by the caller (state += 0x9E3779B97F4A7C15;
  z = state; z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9; z = (z ^ (z >> 27)) * 0x94D049BB133111EB;
  z ^ (z >> 31)), reduced with ``%``.
"""
from __future__ import annotations

import heapq
from typing import List, Sequence, Tuple

MASK64 = (1 << 64) - 1


class SplitMix64:
    def __init__(self, seed: int):
        self.state = seed & MASK64

    def next(self) -> int:
        self.state = (self.state + 0x9E3779B97F4A7C15) & MASK64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
        return z ^ (z >> 31)


def expert_loads(R: Sequence[Sequence[int]]) -> List[int]:
    """``R.sum(axis=0)``."""
    E = len(R[0])
    return [sum(int(R[i][j]) for i in range(len(R))) for j in range(E)]


def replica_allocation(R, N: int, E: int, C: int) -> List[int]:
    """Appendix Alg. 4: every expert starts with one replica; the expert with the highest load per replica
    receives the next one until N*C replicas are handed out."""
    if N * C < E:
        raise ValueError("N*C < E: not every expert can be restored")
    load = expert_loads(R)
    rep = [1] * E
    # max-heap on load/rep; heapq is a min-heap, so the key is negated; the index breaks ties
    pq = [(-(load[j] / rep[j]), j) for j in range(E)]
    heapq.heapify(pq)
    while sum(rep) < N * C:
        _, e = heapq.heappop(pq)
        rep[e] += 1
        heapq.heappush(pq, (-(load[e] / rep[e]), e))
    return rep


def evenly_replicas(N: int, E: int, C: int) -> List[int]:
    base, rem = divmod(N * C, E)
    return [base + (1 if j < rem else 0) for j in range(E)]


def expert_relocation(expert_rep: Sequence[int], loads: Sequence[int], N: int, E: int, C: int, D: int):
    """Alg. 1: replicas in descending order of per-replica load; each goes to the least-loaded eligible
    device among the nodes that hold the fewest replicas of its expert.  Returns A[N][E]."""
    nodes = N // D
    expert_count = [0] * N
    device_loads = [0.0] * N
    A = [[0] * E for _ in range(N)]
    lst: List[Tuple[int, float]] = []
    for j in range(E):
        lst.extend([(j, loads[j] / expert_rep[j])] * expert_rep[j])
    lst.sort(key=lambda t: -t[1])  # stable: equal loads keep expert order
    for expert, load in lst:
        free = [i for i in range(N) if expert_count[i] < C]
        if not free:
            raise ValueError("more replicas than slots")
        fresh = [i for i in free if A[i][expert] == 0]
        eligible = fresh if fresh else free
        node_cnt = [sum(A[i][expert] for i in range(n * D, n * D + D)) for n in range(nodes)]
        cand_nodes = sorted({i // D for i in eligible})
        fewest = min(node_cnt[n] for n in cand_nodes)
        available = [i for i in eligible if node_cnt[i // D] == fewest]
        device = available[0]
        for i in available[1:]:
            if device_loads[i] < device_loads[device]:
                device = i
        A[device][expert] += 1
        device_loads[device] += load
        expert_count[device] += 1
    return A


def lite_routing_rank(R_rank: Sequence[int], A, N: int, E: int, D: int, rank: int) -> List[List[int]]:
    """Appendix Alg. 3 for one device: S[rank][j][k] for all experts j and destinations k."""
    node = rank // D
    S = [[0] * N for _ in range(E)]
    for j in range(E):
        intra = [k for k in range(node * D, node * D + D) for _ in range(A[k][j])]
        everywhere = [k for k in range(N) for _ in range(A[k][j])]
        reps = intra if intra else everywhere
        if not reps:
            if R_rank[j]:
                raise ValueError(f"expert {j} has tokens but no replica")
            continue
        base, rem = divmod(int(R_rank[j]), len(reps))
        for r, k in enumerate(reps):
            S[j][k] += base + (1 if r < rem else 0)
    return S


def lite_routing(R, A, N: int, E: int, D: int):
    """S[i][j][k] for every device i (each device runs Alg. 3 on its own row of R)."""
    return [lite_routing_rank(R[i], A, N, E, D, i) for i in range(N)]


def time_cost(S, N: int, E: int, D: int, v_comm: float, b_intra: float, b_inter: float, v_comp: float,
              b_comp: float, f_ckpt: int) -> Tuple[float, float, float]:
    """Section 4, problem formulation: T = T_comm + T_comp with
    T_comm = 4 V_comm sum_{i,j,k} S[i][j][k] / bw(i,k)   and
    T_comp = (3 + F_ckpt) max_i V_comp sum_{j,k} S[k][j][i] / B_comp.   Returns (T, T_comm, T_comp)."""
    acc = 0.0
    for i in range(N):
        for j in range(E):
            for k in range(N):
                if i == k or S[i][j][k] == 0:
                    continue
                bw = b_intra if i // D == k // D else b_inter
                acc += float(S[i][j][k]) / bw
    t_comm = 4.0 * v_comm * acc
    worst = 0.0
    for i in range(N):
        tokens = 0
        for j in range(E):
            for k in range(N):
                tokens += S[k][j][i]
        t_i = (v_comp * float(tokens)) / b_comp
        if t_i > worst:
            worst = t_i
    t_comp = float(3 + f_ckpt) * worst
    return t_comm + t_comp, t_comm, t_comp


def perturb(rep: Sequence[int], rng: SplitMix64) -> List[int]:
    out = list(rep)
    E = len(out)
    donors = [j for j in range(E) if out[j] > 1]
    if not donors or E < 2:
        return out
    d = donors[rng.next() % len(donors)]
    r = rng.next() % (E - 1)
    if r >= d:
        r += 1
    out[d] -= 1
    out[r] += 1
    return out


def expert_layout(R, N: int, E: int, C: int, D: int, eps: int, seed: int, cost_params: dict):
    """Alg. 2: candidate replica vectors (load-proportional, even, random perturbations of those), each
    placed with Alg. 1, routed with Alg. 3 and priced; the cheapest layout wins (the first one on ties).
    Returns (A, T, index of the winning candidate, list of candidates)."""
    if eps < 1:
        raise ValueError("eps >= 1")
    rng = SplitMix64(seed)
    replicas_set = [replica_allocation(R, N, E, C)]
    if eps >= 2:
        replicas_set.append(evenly_replicas(N, E, C))
    while len(replicas_set) < eps:
        pick = replicas_set[rng.next() % len(replicas_set)]
        replicas_set.append(perturb(pick, rng))
    load = expert_loads(R)
    best_A, best_T, best_idx = None, float("inf"), -1
    for idx, replicas in enumerate(replicas_set):
        A = expert_relocation(replicas, load, N, E, C, D)
        S = lite_routing(R, A, N, E, D)
        T, _, _ = time_cost(S, N, E, D, **cost_params)
        if T < best_T:
            best_A, best_T, best_idx = A, T, idx
    return best_A, best_T, best_idx, replicas_set
