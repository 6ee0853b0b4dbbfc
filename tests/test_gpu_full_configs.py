"""GPU parity at the full benchmark sizes (configurations 3, 4 and 5, and the diffusion-transformer-shaped
share and the load-balanced placement that bench.py --shape dit / zigzag time), in the launch configuration bench.py times: fused ring forward, then
fused ring backward, chunks visited in the ring's order.

The fp64 oracle cannot do these sizes in full, so it does seeded sampled query rows of every head
against ALL keys:
  * run A (dense dO, the benchmark's own run): O, lse and dQ of the sampled rows are exact oracle
    values, because a row's output and dQ depend on that row alone;
  * run B (dO zeroed outside the sampled rows): Delta and dS vanish on every other row, so the
    oracle's dK / dV of the sampled rows are the FULL dK / dV of all keys, and dQ must be exactly
    zero outside the sampled rows.  The kernels do the same work in both runs.
Tolerance: max abs 2e-2 and relative Frobenius 1e-2 per tensor (lse: max abs only)."""
import numpy as np
import pytest
import torch

import paper_2407_00611_amd as st
import synth_inputs as si
from oracle import attention as oa
from util import assert_close, bits_dev, host

pytestmark = pytest.mark.gpu

# workload -> sampled rows per head (configuration 5: the 256 rows its definition names)
CASES = {"cfg3": (lambda: si.paper_workloads()[2], 128), "cfg4": (lambda: si.paper_workloads()[3], 64),
         "cfg5": (lambda: si.paper_workloads()[4], 256), "dit": (si.dit_workload, 64),
         "zigzag": (lambda: si.zigzag_workload(5), 64)}


@pytest.mark.timeout(900)
@pytest.mark.parametrize("cfg", list(CASES))
def test_full_size_sampled_rows(cfg):
    w = CASES[cfg][0]()
    n_rows = CASES[cfg][1]
    G = w.Hq // w.Hkv
    print(f"[{cfg}] generating inputs", flush=True)
    inp = si.make_inputs(w, threads=16, keep_f32=False)
    q = bits_dev(inp.q_bits)
    d_o = bits_dev(inp.d_o_bits)
    ks = [bits_dev(b) for b in inp.k_bits]
    vs = [bits_dev(b) for b in inp.v_bits]
    koffs = [w.k_offset(j) for j in range(w.n_chunks)]
    order, members = st.st_visit_order(w.ring_P, w.ring_C, w.ring_rank)
    if w.q_seg:     # balanced placement: the ring delivers every rank's two pieces of the sequence
        order, members = [c for x in order for c in (x, 2 * w.ring_P - 1 - x)], None
    rows = [si.sampled_rows(w, h, n_rows) for h in range(w.Hq)]

    print(f"[{cfg}] GPU forward + backward, run A (dense dO)", flush=True)
    o, lse, o_low = st.st_ring_fwd(q, ks, vs, w.q_where, koffs, w.causal, w.scale, order, members, st.ST_RING_FUSED)
    dq = torch.zeros_like(o)
    dk = [torch.zeros(k.shape, device="cuda") for k in ks]
    dv = [torch.zeros(k.shape, device="cuda") for k in ks]
    st.st_ring_bwd(q, ks, vs, d_o, o_low, lse, w.q_where, koffs, w.causal, w.scale, order, dq, dk, dv, st.ST_RING_FUSED)
    torch.cuda.synchronize()
    o_s = [host(o[:, torch.from_numpy(rows[h]).cuda(), h]) for h in range(w.Hq)]
    lse_s = [host(lse[:, h, torch.from_numpy(rows[h]).cuda()]) for h in range(w.Hq)]
    dq_s = [host(dq[:, torch.from_numpy(rows[h]).cuda(), h]) for h in range(w.Hq)]
    assert torch.equal(o_low, o.to(torch.bfloat16))
    del dk, dv

    print(f"[{cfg}] GPU backward, run B (dO zero outside the sampled rows)", flush=True)
    keep = torch.zeros((w.B, w.Sq, w.Hq, 1), dtype=torch.bool, device="cuda")
    for h in range(w.Hq):
        keep[:, torch.from_numpy(rows[h]).cuda(), h] = True
    d_o_b = torch.where(keep, d_o, torch.zeros_like(d_o))
    dq_b = torch.zeros_like(o)
    # as bench.py launches the backward: dK / dV assigned (the accumulators start as NaN) and rounded by their kernels
    dk = [torch.full(k.shape, float("nan"), device="cuda") for k in ks]
    dv = [torch.full(k.shape, float("nan"), device="cuda") for k in ks]
    dk_low = [torch.full(k.shape, float("nan"), device="cuda", dtype=torch.bfloat16) for k in ks]
    dv_low = [torch.full(k.shape, float("nan"), device="cuda", dtype=torch.bfloat16) for k in ks]
    st.st_ring_bwd_last(q, ks, vs, d_o_b, o_low, lse, w.q_where, koffs, w.causal, w.scale, order, dq_b, dk, dv,
                        assign=True, dk_lowp=dk_low, dv_lowp=dv_low, mode=st.ST_RING_FUSED)
    torch.cuda.synchronize()
    for j in range(w.n_chunks):
        assert torch.equal(dk_low[j], dk[j].to(torch.bfloat16)) and torch.equal(dv_low[j], dv[j].to(torch.bfloat16)), j
    del dk_low, dv_low
    assert float(torch.where(keep, torch.zeros_like(dq_b), dq_b).abs().max()) == 0.0, "dQ outside the sampled rows"
    for h in range(w.Hq):
        idx = torch.from_numpy(rows[h]).cuda()
        assert torch.equal(dq_b[:, idx, h], dq[:, idx, h]), "a row's dQ must not depend on other rows' dO"
    del o, dq, dq_b, d_o_b, keep

    k_pos = [np.arange(w.Sk, dtype=np.int64) + w.k_offset(j) for j in range(w.n_chunks)]
    for g in range(w.Hkv):
        kg = [si.bf16_bits_to_f32(b[:, :, g:g + 1, :]) for b in inp.k_bits]
        vg = [si.bf16_bits_to_f32(b[:, :, g:g + 1, :]) for b in inp.v_bits]
        dk_ref = [np.zeros((w.B, w.Sk, 1, w.D)) for _ in range(w.n_chunks)]
        dv_ref = [np.zeros((w.B, w.Sk, 1, w.D)) for _ in range(w.n_chunks)]
        for h in range(g * G, (g + 1) * G):
            print(f"[{cfg}] oracle: head {h} ({len(rows[h])} rows x {w.N} keys)", flush=True)
            q_pos = w.q_positions()[rows[h]]
            qh = inp.q[:, rows[h], h:h + 1, :]
            doh = inp.d_o[:, rows[h], h:h + 1, :]
            o_ref, lse_ref = oa.attention_forward(qh, kg, vg, q_pos, k_pos, w.causal, w.scale)
            dq_ref, dk_h, dv_h = oa.attention_backward(qh, kg, vg, doh, q_pos, k_pos, w.causal, w.scale)
            assert_close(o_s[h], o_ref[:, :, 0], "bf16", f"o head {h}")
            assert_close(lse_s[h], lse_ref[:, 0], "bf16", f"lse head {h}", lse=True)
            assert_close(dq_s[h], dq_ref[:, :, 0], "bf16", f"dq head {h}")
            for j in range(w.n_chunks):
                dk_ref[j] += dk_h[j]
                dv_ref[j] += dv_h[j]
        dk_g = np.concatenate([host(dk[j][:, :, g:g + 1]) for j in range(w.n_chunks)], axis=1)
        dv_g = np.concatenate([host(dv[j][:, :, g:g + 1]) for j in range(w.n_chunks)], axis=1)
        assert_close(dk_g, np.concatenate(dk_ref, axis=1), "bf16", f"dk kv head {g} (all chunks)")
        assert_close(dv_g, np.concatenate(dv_ref, axis=1), "bf16", f"dv kv head {g} (all chunks)")
