"""GPU parity, fp32 storage dtype: every C-ABI step against the fp64 oracle, then the whole
share (config 1) in both driver modes.  Tolerance: 1e-5 relative (Frobenius and max-norm)."""
import numpy as np
import pytest
import torch

import paper_2407_00611_amd as st
import synth_inputs as si
from oracle import attention as oa
from util import assert_close, host, positions, upload

pytestmark = pytest.mark.gpu

CASES = [
    # name, B, Hq, Hkv, D, Sq, Sk, n, q_offset, causal
    ("ragged_causal_gqa", 2, 4, 2, 64, 70, 45, 3, 135 - 70, True),
    ("noncausal_d72", 1, 2, 2, 72, 33, 130, 2, 0, False),
    ("causal_future_rows", 1, 2, 1, 8, 37, 20, 2, -5, True),       # first rows see nothing
    ("d256", 1, 1, 1, 256, 9, 67, 1, 100, True),
    ("mid_offset", 1, 3, 1, 32, 64, 64, 4, 100, True),             # chunk 1 diagonal, 2-3 in the future
]


def _workload(c):
    name, B, Hq, Hkv, D, Sq, Sk, n, q0, causal = c
    return si.Workload(name, 70 + len(name), "f32", B, Hq, Hkv, D, Sq, Sk, n, q0, causal, True)


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_block_fwd_merge_delta_bwd_steps(case):
    w = _workload(case)
    inp = si.make_inputs(w)
    q, ks, vs, d_o = upload(inp)
    q_pos, k_pos = positions(w)
    o_acc = torch.zeros((w.B, w.Sq, w.Hq, w.D), device="cuda")
    lse_acc = torch.full((w.B, w.Hq, w.Sq), -float("inf"), device="cuda")
    o_ref, lse_ref = oa.empty_state(w.B, w.Sq, w.Hq, w.D)
    for j in range(w.n_chunks):
        print(f"[{w.name}] block_fwd chunk {j}", flush=True)
        o_p, l_p = st.st_attn_block_fwd(q, ks[j], vs[j], w.q_offset, w.k_offset(j), w.causal, w.scale)
        o_pr, l_pr = oa.block_forward(inp.q, inp.k[j], inp.v[j], q_pos, k_pos[j], w.causal, w.scale)
        assert_close(host(o_p), o_pr, "f32", f"o_part[{j}]")
        assert_close(host(l_p), l_pr, "f32", f"lse_part[{j}]")
        st.st_attn_merge(o_acc, lse_acc, o_p, l_p)
        o_ref, lse_ref = oa.merge(o_ref, lse_ref, o_pr, l_pr)
        assert_close(host(o_acc), o_ref, "f32", f"o_acc after {j}")
        assert_close(host(lse_acc), lse_ref, "f32", f"lse_acc after {j}")
    o_mono, lse_mono = oa.attention_forward(inp.q, inp.k, inp.v, q_pos, k_pos, w.causal, w.scale)
    assert_close(host(o_acc), o_mono, "f32", "o vs monolithic")
    assert_close(host(lse_acc), lse_mono, "f32", "lse vs monolithic")

    delta = st.st_attn_delta(d_o, o_acc)
    assert_close(host(delta), oa.delta(inp.d_o, o_mono), "f32", "delta")

    dq = torch.zeros_like(o_acc)
    dq_ref = np.zeros(o_mono.shape)
    lse_f, delta_f = host(lse_acc), host(delta)
    for j in range(w.n_chunks):
        print(f"[{w.name}] block_bwd chunk {j}", flush=True)
        dk = torch.zeros((w.B, w.Sk, w.Hkv, w.D), device="cuda")
        dv = torch.zeros_like(dk)
        st.st_attn_block_bwd(q, ks[j], vs[j], d_o, lse_acc, delta, w.q_offset, w.k_offset(j), w.causal, w.scale,
                             dq, dk, dv)
        dq_j, dk_r, dv_r = oa.block_backward(inp.q, inp.k[j], inp.v[j], inp.d_o, lse_f, delta_f, q_pos, k_pos[j],
                                             w.causal, w.scale)
        dq_ref += dq_j
        assert_close(host(dk), dk_r, "f32", f"dk[{j}]")
        assert_close(host(dv), dv_r, "f32", f"dv[{j}]")
    assert_close(host(dq), dq_ref, "f32", "dq (steps)")
    dq_m, _, _ = oa.attention_backward(inp.q, inp.k, inp.v, inp.d_o, q_pos, k_pos, w.causal, w.scale)
    assert_close(host(dq), dq_m, "f32", "dq vs monolithic")


def _ring_case(w, order, members, mode):
    inp = si.make_inputs(w)
    q, ks, vs, d_o = upload(inp)
    q_pos, k_pos = positions(w)
    koffs = [w.k_offset(j) for j in range(w.n_chunks)]
    o_acc, lse, o_lowp = st.st_ring_fwd(q, ks, vs, w.q_offset, koffs, w.causal, w.scale, order, members, mode)
    o_ref, lse_ref = oa.attention_forward(inp.q, inp.k, inp.v, q_pos, k_pos, w.causal, w.scale)
    assert_close(host(o_acc), o_ref, "f32", "ring o")
    assert_close(host(lse), lse_ref, "f32", "ring lse")
    assert_close(host(o_lowp), o_ref, "f32", "ring o (storage dtype)")
    dq = torch.zeros_like(o_acc)
    dk = [torch.zeros_like(k) for k in ks]
    dv = [torch.zeros_like(k) for k in ks]
    st.st_ring_bwd(q, ks, vs, d_o, o_lowp, lse, w.q_offset, koffs, w.causal, w.scale, order, dq, dk, dv, mode)
    dq_r, dk_r, dv_r = oa.attention_backward(inp.q, inp.k, inp.v, inp.d_o, q_pos, k_pos, w.causal, w.scale)
    assert_close(host(dq), dq_r, "f32", "ring dq")
    for j in range(w.n_chunks):
        assert_close(host(dk[j]), dk_r[j], "f32", f"ring dk[{j}]")
        assert_close(host(dv[j]), dv_r[j], "f32", f"ring dv[{j}]")


@pytest.mark.parametrize("mode", [st.ST_RING_STEPWISE, st.ST_RING_FUSED], ids=["stepwise", "fused"])
def test_config1_whole_share(mode):
    w = si.paper_workloads()[0]
    for order, members in (([0, 1, 2, 3], None), ([2, 3, 0, 1], [0, 0, 1, 1]), ([3, 1, 2, 0], [0, 1, 2, 3])):
        print(f"[cfg1] mode {mode} order {order}", flush=True)
        _ring_case(w, order, members, mode)


@pytest.mark.parametrize("mode", [st.ST_RING_STEPWISE, st.ST_RING_FUSED], ids=["stepwise", "fused"])
def test_ring_causal_with_concentric_order(mode):
    w = si.Workload("ring_f32_causal", 77, "f32", 1, 4, 2, 64, 48, 48, 16, 15 * 48, True, True)
    order, members = st.st_visit_order(16, 2, 15)
    _ring_case(w, order, members, mode)
    w2 = si.Workload("ring_f32_mid", 78, "f32", 1, 2, 2, 64, 48, 48, 16, 5 * 48, True, True)
    order, members = st.st_visit_order(16, 4, 5)
    _ring_case(w2, order, members, mode)


def test_strided_bhsd_layout_and_empty_chunk():
    w = si.Workload("bhsd", 79, "f32", 2, 2, 1, 64, 40, 24, 1, 0, False, True)
    inp = si.make_inputs(w)
    q, ks, vs, d_o = upload(inp)
    q_bhsd = q.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)          # same values, [B,H,S,D] memory
    k_bhsd = ks[0].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    v_bhsd = vs[0].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    a = st.st_attn_block_fwd(q, ks[0], vs[0], 0, 0, False, w.scale)
    b = st.st_attn_block_fwd(q_bhsd, k_bhsd, v_bhsd, 0, 0, False, w.scale)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    # chunk entirely in the causal future: O = 0, lse = -inf
    o, l = st.st_attn_block_fwd(q, ks[0], vs[0], 0, 1000, True, w.scale)
    assert not o.any() and torch.isneginf(l).all()
    # zero-length chunk
    o, l = st.st_attn_block_fwd(q, ks[0][:, :0], vs[0][:, :0], 0, 0, False, w.scale)
    assert not o.any() and torch.isneginf(l).all()


def test_merge_lowp_output_and_cast():
    torch.manual_seed(0)
    B, Sq, Hq, D = 1, 50, 3, 128
    oa_, ob_ = torch.randn(B, Sq, Hq, D, device="cuda"), torch.randn(B, Sq, Hq, D, device="cuda")
    la, lb = torch.randn(B, Hq, Sq, device="cuda"), torch.randn(B, Hq, Sq, device="cuda")
    la[0, 0, :5] = -float("inf")
    lb[0, 0, 3:8] = -float("inf")
    ref_o, ref_l = oa.merge(host(oa_), host(la), host(ob_), host(lb))
    low = torch.empty(B, Sq, Hq, D, device="cuda", dtype=torch.bfloat16)
    st.st_attn_merge(oa_, la, ob_, lb, st.ST_BF16, low)
    assert_close(host(oa_), ref_o, "f32", "merge o")
    assert_close(host(la), ref_l, "f32", "merge lse")
    assert torch.equal(low, oa_.to(torch.bfloat16))               # RNE, same as torch's conversion
    x = torch.randn(1003, device="cuda")
    assert torch.equal(st.st_cast_from_f32(x, st.ST_BF16), x.to(torch.bfloat16))


def test_merge_ignores_the_o_of_an_empty_state():
    """A state with lse = -inf is the neutral element whatever its O holds (never written, stale, NaN): the
    fold returns the other state.  Reference: the oracle's merge with the empty rows' O set to the neutral 0."""
    torch.manual_seed(1)
    B, Sq, Hq, D = 2, 37, 3, 64
    o_a, o_b = torch.randn(B, Sq, Hq, D, device="cuda"), torch.randn(B, Sq, Hq, D, device="cuda")
    l_a, l_b = torch.randn(B, Hq, Sq, device="cuda"), torch.randn(B, Hq, Sq, device="cuda")
    l_a[0, 0, :9] = -float("inf")        # empty on the accumulator side
    l_b[1, 2, 5:20] = -float("inf")      # empty on the partial side
    l_a[1, 1, 30:] = -float("inf")       # empty on both sides
    l_b[1, 1, 30:] = -float("inf")
    ref_a, ref_b = host(o_a), host(o_b)
    ref_a[np.isneginf(host(l_a)).transpose(0, 2, 1)] = 0.0
    ref_b[np.isneginf(host(l_b)).transpose(0, 2, 1)] = 0.0
    ref_o, ref_l = oa.merge(ref_a, host(l_a), ref_b, host(l_b))
    o_a[torch.isneginf(l_a).transpose(1, 2)] = float("nan")
    o_b[torch.isneginf(l_b).transpose(1, 2)] = float("inf")
    low = torch.empty(B, Sq, Hq, D, device="cuda", dtype=torch.bfloat16)
    st.st_attn_merge(o_a, l_a, o_b, l_b, st.ST_BF16, low)
    assert_close(host(o_a), ref_o, "f32", "merge o")
    assert_close(host(l_a), ref_l, "f32", "merge lse")
    assert not o_a[1, 30:, 1].any()      # empty on both sides: O = 0
    assert torch.equal(low, o_a.to(torch.bfloat16))
