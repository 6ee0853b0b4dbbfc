"""GPU parity of the team-gathered shape at its full size (the workload `bench.py --shape team` times): the
model and layout of configuration 4 (32 / 8 heads of 128, 131072 tokens, P = 32 GPUs in teams of C = 4) as
the last GPU sees it: 16384 gathered query rows, the two gathered team buffers of 16384 tokens it meets,
the 4-way combine that keeps its own 4096 rows, and the backward of the same shape.

The other three members' partial states are computed here by playing those members.  The fp64 oracle does
seeded sampled query rows of every head:
  * the member's partial (O, lse): attention restricted to the keys it met;
  * the combined state (own rows, and all the team's rows): monolithic attention over all 131072 keys;
  * the member's dQ (dense dO): one backward iteration per met buffer with the FINAL lse and Delta;
  * dK / dV of the met buffers: a second backward whose dO is zero outside the sampled rows, so that the
    oracle's contribution of the sampled rows is the whole of it.
Tolerance: max abs 2e-2 and relative Frobenius 1e-2 per tensor (lse: max abs only)."""
import numpy as np
import pytest
import torch

import paper_2407_00611_amd as st
import synth_inputs as si
from oracle import attention as oa
from util import assert_close, bits_dev, host

pytestmark = pytest.mark.gpu

N_ROWS = 48


@pytest.mark.timeout(900)
def test_team_gathered_full_size_sampled_rows():
    w = si.team_workload()
    P, C, rank = w.ring_P, w.ring_C, w.ring_rank
    a_r, n_own = rank % C, w.Sq // C
    G = w.Hq // w.Hkv
    print("[team] generating inputs", flush=True)
    inp = si.make_inputs(w, threads=16, keep_f32=False)
    q, d_o = bits_dev(inp.q_bits), bits_dev(inp.d_o_bits)
    ks = [bits_dev(b) for b in inp.k_bits]
    vs = [bits_dev(b) for b in inp.v_bits]
    koffs = [w.k_offset(j) for j in range(w.n_chunks)]
    rows = [si.sampled_rows(w, h, N_ROWS) for h in range(w.Hq)]
    idx = [torch.from_numpy(r).cuda() for r in rows]

    print("[team] GPU: the four members' partial states, combine", flush=True)
    met = [st.st_team_visit_order(P, C, rank - a_r + a) for a in range(C)]
    assert sorted(j for m in met for j in m) == list(range(w.n_chunks))
    parts = [st.st_ring_fwd(q, ks, vs, w.q_offset, koffs, w.causal, w.scale, met[a], None, st.ST_RING_FUSED,
                            want_lowp=False)[:2] for a in range(C)]
    low = torch.empty((w.B, n_own, w.Hq, w.D), dtype=torch.bfloat16, device="cuda")
    o_own, lse_own = st.st_attn_combine([p[0] for p in parts], [p[1] for p in parts], a_r * n_own, n_own, st.ST_BF16,
                                        o_out_lowp=low)
    o_team, lse_team = st.st_attn_combine([p[0] for p in parts], [p[1] for p in parts])
    torch.cuda.synchronize()
    assert torch.equal(low, o_own.to(torch.bfloat16))
    assert torch.equal(o_own, o_team[:, a_r * n_own:(a_r + 1) * n_own])
    assert torch.equal(lse_own, lse_team[:, :, a_r * n_own:(a_r + 1) * n_own])
    part_o_s = [host(parts[a_r][0][:, idx[h], h]) for h in range(w.Hq)]
    part_l_s = [host(parts[a_r][1][:, h, idx[h]]) for h in range(w.Hq)]
    team_o_s = [host(o_team[:, idx[h], h]) for h in range(w.Hq)]
    team_l_s = [host(lse_team[:, h, idx[h]]) for h in range(w.Hq)]
    o_team_low = o_team.to(torch.bfloat16)
    del parts, o_team, o_own

    mine = met[a_r]
    def grads():
        return (torch.zeros((w.B, w.Sq, w.Hq, w.D), device="cuda"),
                [torch.zeros(ks[j].shape, device="cuda") if j in mine else None for j in range(w.n_chunks)],
                [torch.zeros(ks[j].shape, device="cuda") if j in mine else None for j in range(w.n_chunks)])

    print("[team] GPU backward, run A (dense dO)", flush=True)
    dq, dk, dv = grads()
    st.st_ring_bwd(q, ks, vs, d_o, o_team_low, lse_team, w.q_offset, koffs, w.causal, w.scale, mine, dq, dk, dv,
                   st.ST_RING_FUSED)
    torch.cuda.synchronize()
    dq_s = [host(dq[:, idx[h], h]) for h in range(w.Hq)]
    del dk, dv

    print("[team] GPU backward, run B (dO zero outside the sampled rows)", flush=True)
    keep = torch.zeros((w.B, w.Sq, w.Hq, 1), dtype=torch.bool, device="cuda")
    for h in range(w.Hq):
        keep[:, idx[h], h] = True
    d_o_b = torch.where(keep, d_o, torch.zeros_like(d_o))
    dq_b, dk, dv = grads()
    # as bench.py launches it: dK / dV assigned (the accumulators start as NaN) and rounded by their kernels
    for t in dk + dv:
        if t is not None:
            t.fill_(float("nan"))
    dk_low = [torch.full(t.shape, float("nan"), device="cuda", dtype=torch.bfloat16) if t is not None else None for t in dk]
    dv_low = [torch.full(t.shape, float("nan"), device="cuda", dtype=torch.bfloat16) if t is not None else None for t in dv]
    st.st_ring_bwd_last(q, ks, vs, d_o_b, o_team_low, lse_team, w.q_offset, koffs, w.causal, w.scale, mine, dq_b, dk, dv,
                        assign=True, dk_lowp=dk_low, dv_lowp=dv_low, mode=st.ST_RING_FUSED)
    torch.cuda.synchronize()
    for j in mine:
        assert torch.equal(dk_low[j], dk[j].to(torch.bfloat16)) and torch.equal(dv_low[j], dv[j].to(torch.bfloat16)), j
    del dk_low, dv_low
    assert float(torch.where(keep, torch.zeros_like(dq_b), dq_b).abs().max()) == 0.0, "dQ outside the sampled rows"
    for h in range(w.Hq):
        assert torch.equal(dq_b[:, idx[h], h], dq[:, idx[h], h]), "a row's dQ must not depend on other rows' dO"
    del dq, dq_b, d_o_b, keep

    k_pos = [np.arange(w.Sk, dtype=np.int64) + koffs[j] for j in range(w.n_chunks)]
    for g in range(w.Hkv):
        kg = [si.bf16_bits_to_f32(b[:, :, g:g + 1, :]) for b in inp.k_bits]
        vg = [si.bf16_bits_to_f32(b[:, :, g:g + 1, :]) for b in inp.v_bits]
        dk_ref = {j: np.zeros((w.B, w.Sk, 1, w.D)) for j in mine}
        dv_ref = {j: np.zeros((w.B, w.Sk, 1, w.D)) for j in mine}
        for h in range(g * G, (g + 1) * G):
            print(f"[team] oracle: head {h} ({len(rows[h])} rows x {w.N} keys)", flush=True)
            q_pos = rows[h] + w.q_offset
            qh = inp.q[:, rows[h], h:h + 1, :]
            doh = inp.d_o[:, rows[h], h:h + 1, :]
            o_ref, lse_ref = oa.attention_forward(qh, kg, vg, q_pos, k_pos, w.causal, w.scale)
            o_pr, l_pr = oa.attention_forward(qh, [kg[j] for j in mine], [vg[j] for j in mine], q_pos,
                                              [k_pos[j] for j in mine], w.causal, w.scale)
            assert_close(part_o_s[h], o_pr[:, :, 0], "bf16", f"partial o head {h}")
            assert_close(part_l_s[h], l_pr[:, 0], "bf16", f"partial lse head {h}", lse=True)
            assert_close(team_o_s[h], o_ref[:, :, 0], "bf16", f"combined o head {h}")
            assert_close(team_l_s[h], lse_ref[:, 0], "bf16", f"combined lse head {h}", lse=True)
            delta_ref = oa.delta(doh, o_ref)
            dq_ref = np.zeros_like(o_ref)
            for j in mine:
                dq_j, dk_j, dv_j = oa.block_backward(qh, kg[j], vg[j], doh, lse_ref, delta_ref, q_pos, k_pos[j],
                                                     w.causal, w.scale)
                dq_ref += dq_j
                dk_ref[j] += dk_j
                dv_ref[j] += dv_j
            assert_close(dq_s[h], dq_ref[:, :, 0], "bf16", f"dq head {h} (this member's part)")
        for j in mine:
            assert_close(host(dk[j][:, :, g:g + 1]), dk_ref[j], "bf16", f"dk kv head {g}, buffer {j}")
            assert_close(host(dv[j][:, :, g:g + 1]), dv_ref[j], "bf16", f"dv kv head {g}, buffer {j}")
