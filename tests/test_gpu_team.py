"""GPU parity of the literal per-GPU schedule of the concentric layout (Section 3.2): every GPU holds its
team's gathered queries (C N/P rows), meets one gathered team buffer of keys / values per sub-ring
iteration, and the C members' partial states are combined while each member keeps its own N/P rows
(Algorithm 1, ReduceScatter_combine).  One GPU plays the GPUs of a team one after the other.

Checked against the fp64 oracle: the n-way combine on its own; every member's partial state (attention
restricted to the keys that member met); the combined rows against monolithic attention over the whole
sequence; the backward of the same shape (dQ of the team's rows summed over the members, dK / dV summed
over all teams) against the monolithic gradients."""
import numpy as np
import pytest
import torch

import paper_2407_00611_amd as st
import synth_inputs as si
from oracle import attention as oa
from oracle import visit_order as ov
from util import assert_close, host, upload

pytestmark = pytest.mark.gpu


# ---------------------------------------------------------------------------------- combine on its own

COMBINE_CASES = [
    # n, B, Sq_in, Hq, D, row0, Sq_out
    (1, 1, 40, 2, 128, 0, 40),
    (2, 2, 33, 3, 64, 5, 17),
    (4, 1, 300, 4, 128, 75, 75),
    (5, 1, 130, 1, 8, 0, 130),
    (7, 2, 64, 2, 256, 63, 1),
    (64, 1, 24, 2, 128, 8, 8),
]


@pytest.mark.parametrize("case", COMBINE_CASES, ids=[f"n{c[0]}_D{c[4]}" for c in COMBINE_CASES])
def test_combine_matches_oracle(case):
    n, B, Sq_in, Hq, D, row0, Sq_out = case
    rng = np.random.default_rng(700 + n)
    o_parts = [rng.standard_normal((B, Sq_in, Hq, D)).astype(np.float32) for _ in range(n)]
    l_parts = [(3.0 * rng.standard_normal((B, Hq, Sq_in))).astype(np.float32) for _ in range(n)]
    # empty states: a sprinkling of rows in every state, one state empty throughout, two rows empty everywhere
    for x in range(n):
        empty = rng.random((B, Hq, Sq_in)) < 0.2
        l_parts[x][empty] = -np.inf
        o_parts[x][np.transpose(empty, (0, 2, 1))] = 0.0
    if n > 2:
        l_parts[1][:] = -np.inf
        o_parts[1][:] = 0.0
    for x in range(n):
        l_parts[x][:, :, row0] = -np.inf
        o_parts[x][:, row0] = 0.0
        l_parts[x][:, 0, row0 + Sq_out - 1] = -np.inf
        o_parts[x][:, row0 + Sq_out - 1, 0] = 0.0
    o_ref, l_ref = oa.combine(o_parts, l_parts, row0, Sq_out)
    od = [torch.from_numpy(o).cuda() for o in o_parts]
    ld = [torch.from_numpy(l).cuda() for l in l_parts]
    low = torch.empty((B, Sq_out, Hq, D), dtype=torch.bfloat16, device="cuda")
    o, lse = st.st_attn_combine(od, ld, row0, Sq_out, st.ST_BF16, o_out_lowp=low)
    torch.cuda.synchronize()
    assert_close(host(o), o_ref, "f32", "combine o")
    assert_close(host(lse), l_ref, "f32", "combine lse")
    assert torch.equal(low, o.to(torch.bfloat16))
    assert float(o[:, 0].abs().max()) == 0.0 and bool(torch.isneginf(lse[:, :, 0]).all())
    # fp32 "low precision" copy, and no copy at all
    low32 = torch.empty((B, Sq_out, Hq, D), dtype=torch.float32, device="cuda")
    o2, lse2 = st.st_attn_combine(od, ld, row0, Sq_out, st.ST_F32, o_out_lowp=low32)
    o3, lse3 = st.st_attn_combine(od, ld, row0, Sq_out)
    torch.cuda.synchronize()
    assert torch.equal(o2, o) and torch.equal(low32, o) and torch.equal(o3, o)
    assert torch.equal(lse2, lse) and torch.equal(lse3, lse)


def test_combine_of_two_equals_merge_kernel():
    rng = np.random.default_rng(77)
    o_a, o_b = (torch.from_numpy(rng.standard_normal((1, 50, 2, 128)).astype(np.float32)).cuda() for _ in range(2))
    l_a, l_b = (torch.from_numpy(rng.standard_normal((1, 2, 50)).astype(np.float32)).cuda() for _ in range(2))
    o, lse = st.st_attn_combine([o_a, o_b], [l_a, l_b])
    st.st_attn_merge(o_a, l_a, o_b, l_b)
    torch.cuda.synchronize()
    assert_close(host(o), host(o_a), "f32", "combine vs merge o")
    assert_close(host(lse), host(l_a), "f32", "combine vs merge lse")


# ------------------------------------------------------------------------- the team-gathered schedule

TEAM_CASES = [
    # name, dtype, P, C, n (= N / P tokens per shard), Hq, Hkv, D, causal
    ("p8c2_ragged", "bf16", 8, 2, 88, 2, 1, 128, True),
    ("p8c2_tiles", "bf16", 8, 2, 256, 2, 2, 128, True),
    ("p16c2_full", "bf16", 16, 2, 64, 2, 1, 128, False),
    ("p9c3_d64", "bf16", 9, 3, 96, 2, 1, 64, True),
    ("p16c4_noring", "bf16", 16, 4, 64, 2, 2, 128, True),
    ("p4c1_ring", "bf16", 4, 1, 160, 2, 1, 128, True),
    ("p8c2_f32", "f32", 8, 2, 40, 2, 1, 64, True),
]


def _sequence(case):
    """The whole sequence as one workload: Q / dO of all N rows, K / V as the P / C gathered team buffers."""
    name, dtype, P, C, n, Hq, Hkv, D, causal = case
    w = si.Workload(f"team_{name}", 95, dtype, 1, Hq, Hkv, D, P * n, C * n, P // C, 0, causal, True)
    return w, si.make_inputs(w, threads=4)


@pytest.mark.parametrize("mode", [st.ST_RING_FUSED, st.ST_RING_STEPWISE], ids=["fused", "stepwise"])
@pytest.mark.parametrize("case", TEAM_CASES, ids=[c[0] for c in TEAM_CASES])
def test_team_gathered_forward_and_backward(case, mode):
    name, dtype, P, C, n, Hq, Hkv, D, causal = case
    w, inp = _sequence(case)
    q_all, ks, vs, do_all = upload(inp)
    team_rows = C * n
    koffs = [w.k_offset(j) for j in range(w.n_chunks)]
    k_pos = [np.arange(w.Sk, dtype=np.int64) + koffs[j] for j in range(w.n_chunks)]
    q_pos_all = np.arange(w.Sq, dtype=np.int64)
    o_ref, lse_ref = oa.attention_forward(inp.q, inp.k, inp.v, q_pos_all, k_pos, causal, w.scale)
    dq_ref, dk_ref, dv_ref = oa.attention_backward(inp.q, inp.k, inp.v, inp.d_o, q_pos_all, k_pos, causal, w.scale)

    dq_all = torch.zeros((1, w.Sq, Hq, D), dtype=torch.float32, device="cuda")
    dk = [torch.zeros(k.shape, dtype=torch.float32, device="cuda") for k in ks]
    dv = [torch.zeros(k.shape, dtype=torch.float32, device="cuda") for k in ks]
    for t in range(P // C):
        r0 = t * team_rows
        q_team = q_all[:, r0:r0 + team_rows]
        do_team = do_all[:, r0:r0 + team_rows]
        parts = []
        for a in range(C):
            buffers = st.st_team_visit_order(P, C, t * C + a)
            assert buffers == ov.team_visit_order(P, C, t * C + a)
            o_p, l_p, _ = st.st_ring_fwd(q_team, ks, vs, r0, koffs, causal, w.scale, buffers, None, mode, want_lowp=False)
            parts.append((o_p, l_p, buffers))
            # the member's partial state: attention of the team's rows over the keys this member met
            o_pr, l_pr = oa.attention_forward(inp.q[:, r0:r0 + team_rows], [inp.k[j] for j in buffers],
                                              [inp.v[j] for j in buffers], q_pos_all[r0:r0 + team_rows],
                                              [k_pos[j] for j in buffers], causal, w.scale)
            torch.cuda.synchronize()
            assert_close(host(o_p), o_pr, dtype, f"team {t} member {a}: partial o")
            assert_close(host(l_p), l_pr, dtype, f"team {t} member {a}: partial lse", lse=True)
        # combine: member a keeps its own n rows
        for a in range(C):
            low = torch.empty((1, n, Hq, D), dtype=q_all.dtype, device="cuda")
            o_f, l_f = st.st_attn_combine([p[0] for p in parts], [p[1] for p in parts], a * n, n,
                                          st.ST_BF16 if dtype == "bf16" else st.ST_F32, o_out_lowp=low)
            torch.cuda.synchronize()
            rows = slice(r0 + a * n, r0 + (a + 1) * n)
            assert_close(host(o_f), o_ref[:, rows], dtype, f"rank {t * C + a}: o")
            assert_close(host(l_f), lse_ref[:, :, rows], dtype, f"rank {t * C + a}: lse", lse=True)
            assert torch.equal(low, o_f.to(q_all.dtype))
        # backward of the same shape: the team's final O and lse (all C n rows), every member against its buffers
        o_team, l_team = st.st_attn_combine([p[0] for p in parts], [p[1] for p in parts])
        o_team_low = o_team.to(q_all.dtype)
        dq_team = torch.zeros((1, team_rows, Hq, D), dtype=torch.float32, device="cuda")
        for a in range(C):
            st.st_ring_bwd(q_team, ks, vs, do_team, o_team_low, l_team, r0, koffs, causal, w.scale, parts[a][2],
                           dq_team, dk, dv, mode)
        dq_all[:, r0:r0 + team_rows] = dq_team
    torch.cuda.synchronize()
    assert_close(host(dq_all), dq_ref, dtype, "dq (summed over the members of each team)")
    for j in range(w.n_chunks):
        assert_close(host(dk[j]), dk_ref[j], dtype, f"dk buffer {j} (summed over all teams)")
        assert_close(host(dv[j]), dv_ref[j], dtype, f"dv buffer {j} (summed over all teams)")
