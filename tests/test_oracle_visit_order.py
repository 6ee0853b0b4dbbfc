"""Pins for the visit-order oracle (CPU only): the paper's stated counts, hand
evaluations of the two appendix algorithms, and coverage invariants."""
import os

import pytest

from oracle import visit_order as ov

GOLD = {}
with open(os.path.join(os.path.dirname(__file__), "golden", "visit_order_paper.txt")) as f:
    for line in f:
        if line.strip() and not line.startswith("#"):
            key, val = line.split("=")
            GOLD[key.strip()] = [int(x) for x in val.split()]


def test_paper_counts():
    assert len(ov.sub_rings(8, 2)) == GOLD["P8_C2_subrings"][0]
    for key, val in GOLD.items():
        if key.endswith("_iterations"):
            P, C = int(key.split("_")[0][1:]), int(key.split("_")[1][1:])
            held = ov.simulate_cluster(P, C)
            assert len(held) == val[0]
            assert all(len(r) == val[0] for r in ov.sub_rings(P, C))


def test_hand_evaluated_maps():
    assert [ov.get_init_send(g // 2, g % 2, 4, 2) for g in range(8)] == GOLD["P8_C2_init_send"]
    assert [ov.get_p2p_config(g // 2, g % 2, 4, 2)[0] for g in range(8)] == GOLD["P8_C2_next"]
    # with two GPUs per sub-ring, next and last coincide
    assert all(ov.get_p2p_config(g // 2, g % 2, 4, 2)[0] == ov.get_p2p_config(g // 2, g % 2, 4, 2)[1]
               for g in range(8))
    assert ov.sub_rings(8, 2) == [[0, 2], [1, 3], [4, 6], [5, 7]]
    # four GPUs per sub-ring: next and last differ, both outputs of the algorithm are pinned
    assert [ov.get_p2p_config(g // 2, g % 2, 8, 2)[0] for g in range(16)] == GOLD["P16_C2_next"]
    assert [ov.get_p2p_config(g // 2, g % 2, 8, 2)[1] for g in range(16)] == GOLD["P16_C2_last"]
    assert [ov.get_p2p_config(g, 0, 16, 1)[1] for g in range(16)] == GOLD["P16_C1_last"]


@pytest.mark.parametrize("P,C", [(4, 1), (8, 2), (16, 2), (32, 2), (64, 4), (36, 3), (27, 3)])
def test_last_is_the_inverse_of_next(P, C):
    """A GPU receives from the GPU that sends to it: last(next(g)) = g = next(last(g)) for every rank."""
    d_a, d_t = C, P // C
    nxt = [ov.get_p2p_config(g // C, g % C, d_t, d_a)[0] for g in range(P)]
    lst = [ov.get_p2p_config(g // C, g % C, d_t, d_a)[1] for g in range(P)]
    assert sorted(nxt) == list(range(P)) and sorted(lst) == list(range(P))
    assert all(lst[nxt[g]] == g and nxt[lst[g]] == g for g in range(P))


@pytest.mark.parametrize("P,C", [(1, 1), (4, 1), (4, 2), (8, 2), (16, 1), (16, 2), (16, 4), (32, 4),
                                 (32, 2), (64, 4), (64, 8), (36, 3), (18, 3)])
def test_coverage_invariants(P, C):
    held = ov.simulate_cluster(P, C)
    S = P // (C * C)
    assert len(held) == S
    for g0 in range(0, P, C):                     # one team
        seen = []
        for a in range(C):
            mine = [held[i][g0 + a] for i in range(S)]
            assert len(set(mine)) == S            # a member never meets a buffer twice
            seen += mine
        assert sorted(seen) == list(range(P // C))    # team covers every team buffer once
    for i in range(S):                            # within a sub-ring no two GPUs hold the same buffer
        for ring in ov.sub_rings(P, C):
            assert len({held[i][g] for g in ring}) == len(ring)
    for rank in range(P):
        shards, members = ov.visit_order(P, C, rank)
        assert sorted(shards) == list(range(P))
        assert members == sorted(members) and set(members) == set(range(C))
        assert all(members.count(a) == P // C for a in range(C))


def test_team_order_is_the_member_part_of_the_shard_order():
    """The literal schedule (team buffers met by one GPU) and the one-GPU rendering used for a single shard
    (all C members in turn, buffers expanded to shards) describe the same walk."""
    for P, C in [(8, 2), (16, 2), (32, 4), (64, 4), (36, 3), (16, 1)]:
        S = P // (C * C)
        for rank in range(P):
            buffers = ov.team_visit_order(P, C, rank)
            assert len(buffers) == S and len(set(buffers)) == S
            assert all(b % C == rank % C for b in buffers)          # member a only meets buffers = a (mod C)
            shards, members = ov.visit_order(P, C, rank)
            mine = [s for s, m in zip(shards, members) if m == rank % C]
            assert mine == [b * C + c for b in buffers for c in range(C)]
        # the C members of a team meet every team buffer exactly once between them
        for t0 in range(0, P, C):
            seen = sorted(b for a in range(C) for b in ov.team_visit_order(P, C, t0 + a))
            assert seen == list(range(P // C))


def test_c1_is_the_plain_ring():
    # Ring attention: rank r starts on its own shard and then receives from its predecessor
    for P, r in [(4, 0), (8, 3), (16, 15)]:
        shards, members = ov.visit_order(P, 1, r)
        assert shards == [(r - i) % P for i in range(P)]
        assert members == [0] * P


def test_c_sqrt_p_has_one_iteration_per_member():
    shards, members = ov.visit_order(16, 4, 5)
    assert members == [a for a in range(4) for _ in range(4)]
    for a in range(4):
        blk = shards[4 * a:4 * a + 4]
        assert blk == list(range(blk[0], blk[0] + 4)) and blk[0] % 4 == 0


def test_invalid_layouts_are_rejected():
    for P, C in [(8, 3), (8, 4), (0, 1), (8, 0), (12, 4)]:
        with pytest.raises(ValueError):
            ov.visit_order(P, C, 0)
    with pytest.raises(ValueError):
        ov.visit_order(8, 2, 8)
