"""CPU oracle for the communication one attention block forward implies, per GPU.

TEST INFRASTRUCTURE ONLY; shares no code with the library and is never
imported by it.

Section 3.2 "Theoretical Analysis" gives three expressions (ring attention's
P2P, the concentric layout's collectives, the concentric layout's P2P); their
volume terms are counted here, and the times follow from a bandwidth W
(bytes per second) and a latency L (seconds) charged once per ring step.
Instead of evaluating the closed forms, this module lists every message one
GPU sends and adds up the bytes, with Python integers:

  * ring attention: in each of the P - 1 steps the GPU passes on the K shard
    and the V shard it holds (N / P tokens each);
  * concentric layout, collectives: a ring all-gather over the C team members
    of Q, K and V forwards one shard per tensor in each of its C - 1 steps, and
    the reduce-scatter of O sends one shard-sized piece in each of its C - 1
    steps;
  * concentric layout, P2P: a sub-ring has P / C^2 GPUs (taken from the
    cluster simulation in oracle.visit_order); in each of its steps but the last
    the GPU passes on the gathered K and V of a team (C N / P tokens each).

Reading: a shard of one tensor is B * (N / P) * H elements of `e` bytes; the
initial placement send that precedes the sub-ring loop is not part of the
paper's three expressions and is not counted.
"""
from __future__ import annotations

from typing import Dict, List, Tuple

from oracle import visit_order as ov


def shard_bytes(B: int, N: int, H: int, P: int, e: int) -> int:
    if N % P:
        raise ValueError("P must divide N")
    return B * (N // P) * H * e


def ring_messages(P: int, B: int, N: int, H: int, e: int) -> List[Tuple[str, int]]:
    """(what, bytes) of every message one GPU sends in plain ring attention."""
    s = shard_bytes(B, N, H, P, e)
    out = []
    for step in range(P - 1):
        out.append((f"step {step}: K shard", s))
        out.append((f"step {step}: V shard", s))
    return out


def startrail_collective_messages(P: int, C: int, B: int, N: int, H: int, e: int) -> List[Tuple[str, int]]:
    ov.check_layout(P, C)
    s = shard_bytes(B, N, H, P, e)
    out = []
    for tensor in ("Q", "K", "V"):
        for step in range(C - 1):
            out.append((f"all-gather {tensor}, step {step}", s))
    for step in range(C - 1):
        out.append((f"reduce-scatter O, step {step}", s))
    return out


def startrail_p2p_messages(P: int, C: int, B: int, N: int, H: int, e: int) -> List[Tuple[str, int]]:
    ov.check_layout(P, C)
    s = shard_bytes(B, N, H, P, e)
    ring_len = len(ov.sub_rings(P, C)[0])
    out = []
    for step in range(ring_len - 1):
        for tensor in ("K", "V"):
            for member in range(C):                      # the C shards a team gathered travel together
                out.append((f"sub-ring step {step}: {tensor} shard of member {member}", s))
    return out


def report(P: int, C: int, B: int, N: int, H: int, e: int, W: float = 1.0, L: float = 0.0) -> Dict[str, float]:
    ring = ring_messages(P, B, N, H, e)
    coll = startrail_collective_messages(P, C, B, N, H, e)
    p2p = startrail_p2p_messages(P, C, B, N, H, e)
    ring_iters = len(ring) // 2
    st_iters = len(p2p) // (2 * C)
    # one ring step = its messages back to back on the link, plus one latency; the paper charges the
    # collectives no latency
    ring_time = sum(sum(b for _, b in ring[2 * i:2 * i + 2]) / W + L for i in range(ring_iters))
    p2p_time = sum(sum(b for _, b in p2p[2 * C * i:2 * C * (i + 1)]) / W + L for i in range(st_iters))
    coll_time = sum(b for _, b in coll) / W
    return {
        "ring_iterations": ring_iters,
        "startrail_iterations": st_iters,
        "ring_p2p_bytes_per_iter": sum(b for _, b in ring[:2]) if ring else 2 * shard_bytes(B, N, H, P, e),
        "startrail_p2p_bytes_per_iter": sum(b for _, b in p2p[:2 * C]) if p2p else 2 * C * shard_bytes(B, N, H, P, e),
        "ring_p2p_bytes": sum(b for _, b in ring),
        "startrail_p2p_bytes": sum(b for _, b in p2p),
        "startrail_collective_bytes": sum(b for _, b in coll),
        "ring_p2p_seconds": ring_time,
        "startrail_p2p_seconds": p2p_time,
        "startrail_collective_seconds": coll_time,
    }
