"""CPU oracle for the chunk-visit order of the concentric-ring schedule.

TEST INFRASTRUCTURE ONLY; shares no code with the library and is never
imported by it.

It *simulates the whole cluster* as the paper describes it (Section 3.2
"Forward Propagation"; appendix algorithms get_init_send and get_P2P_config):
P GPUs in teams of C, every member of team t holds the team's gathered KV
(sequence shards t*C .. t*C+C-1) after the all-gather; each GPU sends that
buffer to its initial target; then for P/C^2 iterations every GPU computes on
the buffer it holds and passes it to the next GPU of its sub-ring.  The
order in which the C members of one team meet the sequence shards is read
off the simulation.

Readings where the text leaves room: global rank = r_t * C + r_a; the two
divisions in the appendix algorithms are integer floor divisions; ``%`` is
the non-negative (floor) modulus; C must satisfy C >= 1 and C*C | P.
"""
from __future__ import annotations

from typing import List, Tuple


def check_layout(P: int, C: int) -> None:
    if P < 1 or C < 1 or P % (C * C) != 0:
        raise ValueError(f"need C >= 1 and C*C | P, got P={P}, C={C}")


def get_init_send(r_t: int, r_a: int, d_t: int, d_a: int) -> int:
    """Appendix algorithm get_init_send: global rank that receives the team KV
    of GPU (r_t, r_a) before the loop."""
    team_group_size = d_t // d_a
    target_team_group_rank = r_a
    target_team = target_team_group_rank * team_group_size + r_t // d_a
    target_intra = r_t % d_a
    return target_team * d_a + target_intra


def get_p2p_config(r_t: int, r_a: int, d_t: int, d_a: int) -> Tuple[int, int]:
    """Appendix algorithm get_P2P_config: (next, last) global ranks in the sub-ring."""
    team_group_size = d_t // d_a
    self_group = r_t // team_group_size
    next_team = (r_t + 1) % team_group_size + team_group_size * self_group
    last_team = (r_t - 1) % team_group_size + team_group_size * self_group   # Python % is floor-mod
    return r_a + next_team * d_a, r_a + last_team * d_a


def simulate_cluster(P: int, C: int) -> List[List[int]]:
    """held[i][g] = index of the team KV buffer GPU g computes on at iteration i
    (i = 0 .. P/C^2 - 1).  Buffer tau is the gathered KV of team tau."""
    check_layout(P, C)
    d_a, d_t = C, P // C
    iters = P // (C * C)
    start = [g // C for g in range(P)]                 # after the all-gather
    cur = [None] * P
    for g in range(P):                                  # initial dispatch
        cur[get_init_send(g // C, g % C, d_t, d_a)] = start[g]
    assert all(x is not None for x in cur), "initial dispatch is not a permutation"
    held = []
    for _ in range(iters):
        held.append(list(cur))
        nxt = [None] * P
        for g in range(P):
            n, _last = get_p2p_config(g // C, g % C, d_t, d_a)
            nxt[n] = cur[g]
        cur = nxt
    return held


def sub_rings(P: int, C: int) -> List[List[int]]:
    """The disjoint sub-rings (as sorted rank lists) that get_P2P_config induces."""
    check_layout(P, C)
    d_a, d_t = C, P // C
    seen, rings = set(), []
    for g in range(P):
        if g in seen:
            continue
        ring, x = [], g
        while x not in ring:
            ring.append(x)
            x = get_p2p_config(x // C, x % C, d_t, d_a)[0]
        seen.update(ring)
        rings.append(sorted(ring))
    return rings


def visit_order(P: int, C: int, rank: int) -> Tuple[List[int], List[int]]:
    """Order in which the query shard of ``rank`` meets the P sequence shards
    when one GPU plays all C members of the rank's team in turn.

    Returns (shard_idx, member_of), both of length P: member a' = 0..C-1 walks
    its P/C^2 iterations; each iteration's buffer expands to its C shards in
    ascending order.  ``member_of`` tells which member's running state a shard
    folds into."""
    check_layout(P, C)
    if not 0 <= rank < P:
        raise ValueError("rank out of range")
    held = simulate_cluster(P, C)
    t = rank // C
    shard_idx, member_of = [], []
    for a in range(C):
        g = t * C + a
        for i in range(len(held)):
            tau = held[i][g]
            for c in range(C):
                shard_idx.append(tau * C + c)
                member_of.append(a)
    return shard_idx, member_of


def team_visit_order(P: int, C: int, rank: int) -> List[int]:
    """Team buffers GPU ``rank`` computes on, one per sub-ring iteration, read off
    the cluster simulation (Section 3.2: the literal schedule, in which every GPU
    holds its team's C N/P queries and meets one gathered team buffer per iteration)."""
    check_layout(P, C)
    if not 0 <= rank < P:
        raise ValueError("rank out of range")
    return [row[rank] for row in simulate_cluster(P, C)]
