"""CPU oracle of the token dispatcher: the lite routing of the paper's appendix (Lite Routing Algorithm)
applied pair by pair, fused with the stable permutation of the rows.

TEST INFRASTRUCTURE ONLY (plain Python loops); only ``tests/`` imports it; shares nothing with the HIP path.

The appendix fixes *how many* of a device's tokens for expert j go to each replica (an even split over
the replicas in the sender's node, or over all replicas if the node has none).  Which token goes where is
not fixed; the reading taken here (and by the kernels): the tokens of expert j, in their stable order
(pair index p = t*k + s ascending), are cut into consecutive blocks, one per replica, the replicas in
ascending (device, slot) order, the larger blocks first.  A replica slot is a "group"; groups are numbered
by (device, then expert index on that device, then copy), and the permuted rows are ordered by group, so
the rows bound for one device are contiguous (one All-to-All send region per device).
"""
from __future__ import annotations

from typing import List, Sequence, Tuple


def dispatch_table(A: Sequence[Sequence[int]], N: int, E: int, D: int, rank: int):
    """Groups of a layout and the replicas device `rank` may use for each expert.

    Returns (G, expert_of_group[G], device_of_group[G], rep_begin[E+1], rep_group[...]): the groups of expert j
    that `rank` routes to are rep_group[rep_begin[j]:rep_begin[j+1]], in ascending group order: the replicas
    inside rank's node if there are any, else all replicas (appendix, Lite Routing Algorithm)."""
    expert_of_group: List[int] = []
    device_of_group: List[int] = []
    for i in range(N):
        for j in range(E):
            for _ in range(A[i][j]):
                expert_of_group.append(j)
                device_of_group.append(i)
    G = len(expert_of_group)
    node = rank // D
    rep_begin, rep_group = [0], []
    for j in range(E):
        mine = [g for g in range(G) if expert_of_group[g] == j]
        intra = [g for g in mine if device_of_group[g] // D == node]
        rep_group.extend(intra if intra else mine)
        rep_begin.append(len(rep_group))
    return G, expert_of_group, device_of_group, rep_begin, rep_group


def permute_lite(ids: Sequence[Sequence[int]], E: int, G: int, rep_begin: Sequence[int], rep_group: Sequence[int]):
    """ids[T][k] -> (expert_counts[E], group_counts[G], group_offsets[G+1], row_of_pair[R], pair_of_row[R])."""
    T, k = len(ids), len(ids[0])
    R = T * k
    pairs_of: List[List[int]] = [[] for _ in range(E)]
    for p in range(R):
        pairs_of[ids[p // k][p % k]].append(p)          # stable: ascending pair index
    expert_counts = [len(v) for v in pairs_of]
    group_counts = [0] * G
    group_of_pair = [-1] * R
    for j in range(E):
        reps = rep_group[rep_begin[j]:rep_begin[j + 1]]
        n = expert_counts[j]
        if n == 0:
            continue
        if not reps:
            raise ValueError(f"expert {j} has tokens but no replica")
        base, rem = divmod(n, len(reps))
        q = 0
        for r, g in enumerate(reps):
            share = base + (1 if r < rem else 0)
            for p in pairs_of[j][q:q + share]:
                group_of_pair[p] = g
            group_counts[g] += share
            q += share
    group_offsets = [0]
    for g in range(G):
        group_offsets.append(group_offsets[-1] + group_counts[g])
    nxt = list(group_offsets[:G])
    row_of_pair = [0] * R
    pair_of_row = [0] * R
    for p in range(R):                                   # stable inside a group as well
        g = group_of_pair[p]
        row_of_pair[p] = nxt[g]
        pair_of_row[nxt[g]] = p
        nxt[g] += 1
    return expert_counts, group_counts, group_offsets, row_of_pair, pair_of_row
