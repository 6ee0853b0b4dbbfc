"""GPU parity, bf16 backward (MFMA path) against the fp64 oracle on the bf16-rounded inputs.
Tolerance: max abs 2e-2 and relative Frobenius 1e-2 per tensor."""

import numpy as np
import pytest
import torch

import paper_2407_00611_amd as st
import synth_inputs as si
from oracle import attention as oa
from util import assert_close, assert_close_wide, host, launcher_switch, positions, upload

pytestmark = pytest.mark.gpu

STEP_CASES = [
    # name, B, Hq, Hkv, D, Sq, Sk, n, q_offset, causal
    ("ragged_causal_gqa_d128", 2, 4, 2, 128, 300, 200, 3, 600 - 300, True),
    ("noncausal_d128", 1, 2, 2, 128, 70, 130, 2, 0, False),
    ("future_rows_d128", 1, 2, 1, 128, 100, 90, 2, -37, True),
    ("ragged_causal_d64", 2, 3, 1, 64, 260, 150, 2, 40, True),
    ("noncausal_d64", 1, 4, 4, 64, 515, 64, 3, 0, False),
    ("one_row_one_key", 1, 1, 1, 128, 1, 1, 1, 0, True),
    ("wide_kv_tile", 1, 2, 1, 128, 130, 600, 1, 450, True),
    # head_dim 128 with full 256-key tiles: the hand-scheduled dK/dV loop takes the fully visible 32-row blocks
    ("fast_one_block", 1, 2, 2, 128, 32, 256, 1, 0, False),
    ("fast_gqa_two_tiles", 2, 4, 2, 128, 160, 512, 2, 700, True),
    ("fast_three_heads_ragged", 1, 3, 1, 128, 103, 296, 2, 1000, True),
    ("fast_long_run", 1, 2, 1, 128, 416, 256, 2, 256, True),
    # full 256-query tiles: the hand-scheduled dQ loop takes the fully visible 64-key tiles of every chunk
    ("dq_fast_one_tile", 1, 1, 1, 128, 256, 64, 1, 0, False),
    ("dq_fast_two_tiles", 1, 1, 1, 128, 256, 128, 1, 0, False),
    ("dq_fast_chunk_switches", 2, 4, 2, 128, 300, 320, 3, 0, False),
    ("dq_fast_causal_mix", 1, 2, 1, 128, 512, 200, 5, 520, True),
    # the same loops generated for head size 64
    ("dq_fast64_one_tile", 1, 1, 1, 64, 256, 64, 1, 0, False),
    ("dq_fast64_two_tiles", 1, 1, 1, 64, 256, 128, 1, 0, False),
    ("dq_fast64_chunk_switches", 2, 4, 2, 64, 300, 320, 3, 0, False),
    ("dq_fast64_causal_mix", 1, 2, 1, 64, 512, 200, 5, 520, True),
    ("dq_fast64_long", 1, 3, 3, 64, 256, 1024, 3, 0, False),
    ("fast64_one_block", 1, 2, 2, 64, 32, 256, 1, 0, False),
    ("fast64_gqa_two_tiles", 2, 4, 2, 64, 160, 512, 2, 700, True),
    ("fast64_three_heads_ragged", 1, 3, 1, 64, 103, 296, 2, 1000, True),
    ("fast64_long_run", 1, 2, 1, 64, 416, 256, 2, 256, True),
]


def _workload(c):
    name, B, Hq, Hkv, D, Sq, Sk, n, q0, causal = c
    return si.Workload(name, 90 + len(name), "bf16", B, Hq, Hkv, D, Sq, Sk, n, q0, causal, True)


@pytest.mark.parametrize("case", STEP_CASES, ids=[c[0] for c in STEP_CASES])
def test_delta_and_block_bwd_steps(case):
    w = _workload(case)
    inp = si.make_inputs(w)
    q, ks, vs, d_o = upload(inp)
    q_pos, k_pos = positions(w)
    # final statistics from the oracle, so that this test isolates the backward step
    o_ref, lse_ref = oa.attention_forward(inp.q, inp.k, inp.v, q_pos, k_pos, w.causal, w.scale)
    o_dev = torch.from_numpy(o_ref.astype(np.float32)).cuda()
    lse_dev = torch.from_numpy(lse_ref.astype(np.float32)).cuda()
    delta = st.st_attn_delta(d_o, o_dev)
    delta_ref = oa.delta(inp.d_o, o_ref)
    assert_close(host(delta), delta_ref, "bf16", "delta")
    o_bf = o_dev.to(torch.bfloat16)                                     # O saved in the storage dtype
    delta_bf = st.st_attn_delta(d_o, o_bf)
    assert_close(host(delta_bf), oa.delta(inp.d_o, host(o_bf)), "bf16", "delta from bf16 O")

    dq = torch.zeros((w.B, w.Sq, w.Hq, w.D), device="cuda")
    dq_ref = np.zeros(o_ref.shape)
    lse_f, delta_f = host(lse_dev), host(delta)
    for j in range(w.n_chunks):
        print(f"[{w.name}] block_bwd chunk {j}", flush=True)
        dk = torch.zeros((w.B, w.Sk, w.Hkv, w.D), device="cuda")
        dv = torch.zeros_like(dk)
        st.st_attn_block_bwd(q, ks[j], vs[j], d_o, lse_dev, delta, w.q_offset, w.k_offset(j), w.causal, w.scale,
                             dq, dk, dv)
        dq_j, dk_r, dv_r = oa.block_backward(inp.q, inp.k[j], inp.v[j], inp.d_o, lse_f, delta_f, q_pos, k_pos[j],
                                             w.causal, w.scale)
        dq_ref += dq_j
        assert_close(host(dk), dk_r, "bf16", f"dk[{j}]")
        assert_close(host(dv), dv_r, "bf16", f"dv[{j}]")
    assert_close(host(dq), dq_ref, "bf16", "dq (steps)")
    dq_m, _, _ = oa.attention_backward(inp.q, inp.k, inp.v, inp.d_o, q_pos, k_pos, w.causal, w.scale)
    assert_close(host(dq), dq_m, "bf16", "dq vs monolithic")


@pytest.mark.parametrize("D", [128, 64])
def test_block_bwd_with_and_without_workspace(D):
    """The step call takes an optional workspace for the scaled copy of Q.  With it the hand-scheduled dK/dV loop
    runs, without it the general kernel computes the same blocks from the same operands: both match the oracle,
    and dQ (the same kernels either way) is bit-identical."""
    w = si.Workload(f"block_ws_d{D}", 93, "bf16", 1, 4, 2, D, 320, 512, 1, 600, True, True)
    inp = si.make_inputs(w)
    q, ks, vs, d_o = upload(inp)
    q_pos, k_pos = positions(w)
    o_ref, lse_ref = oa.attention_forward(inp.q, inp.k, inp.v, q_pos, k_pos, w.causal, w.scale)
    lse_dev = torch.from_numpy(lse_ref.astype(np.float32)).cuda()
    delta = st.st_attn_delta(d_o, torch.from_numpy(o_ref.astype(np.float32)).cuda())
    dq_r, dk_r, dv_r = oa.block_backward(inp.q, inp.k[0], inp.v[0], inp.d_o, host(lse_dev), host(delta), q_pos, k_pos[0],
                                         w.causal, w.scale)
    need = st.st_attn_block_bwd_workspace_bytes(q, ks[0], w.q_offset, 0, w.causal, w.scale)
    assert need >= q.numel() * 2
    out = []
    for ws in (None, False, torch.empty(need + 256, dtype=torch.uint8, device="cuda")):
        dq = torch.zeros((w.B, w.Sq, w.Hq, w.D), device="cuda")
        dk = torch.zeros((w.B, w.Sk, w.Hkv, w.D), device="cuda")
        dv = torch.zeros_like(dk)
        print(f"[{w.name}] workspace {'none' if ws is False else 'given'}", flush=True)
        st.st_attn_block_bwd(q, ks[0], vs[0], d_o, lse_dev, delta, w.q_offset, 0, w.causal, w.scale, dq, dk, dv, workspace=ws)
        torch.cuda.synchronize()
        assert_close(host(dq), dq_r, "bf16", "dq")
        assert_close(host(dk), dk_r, "bf16", "dk")
        assert_close(host(dv), dv_r, "bf16", "dv")
        out.append((dq, dk, dv))
    assert torch.equal(out[0][0], out[1][0]) and torch.equal(out[0][0], out[2][0])
    assert torch.equal(out[0][1], out[2][1]) and torch.equal(out[0][2], out[2][2])
    with pytest.raises(st.StarTrailError):
        st.st_attn_block_bwd(q, ks[0], vs[0], d_o, lse_dev, delta, w.q_offset, 0, w.causal, w.scale, *out[0],
                             workspace=torch.empty(1024, dtype=torch.uint8, device="cuda"))


def _ring_fwd_bwd(w, order, members, mode):
    inp = si.make_inputs(w)
    q, ks, vs, d_o = upload(inp)
    q_pos, k_pos = positions(w)
    koffs = [w.k_offset(j) for j in range(w.n_chunks)]
    o, lse, o_low = st.st_ring_fwd(q, ks, vs, w.q_offset, koffs, w.causal, w.scale, order, members, mode)
    dq = torch.zeros_like(o)
    dk = [torch.zeros(k.shape, device="cuda") for k in ks]
    dv = [torch.zeros(k.shape, device="cuda") for k in ks]
    st.st_ring_bwd(q, ks, vs, d_o, o_low, lse, w.q_offset, koffs, w.causal, w.scale, order, dq, dk, dv, mode)
    torch.cuda.synchronize()
    o_ref, lse_ref = oa.attention_forward(inp.q, inp.k, inp.v, q_pos, k_pos, w.causal, w.scale)
    dq_r, dk_r, dv_r = oa.attention_backward(inp.q, inp.k, inp.v, inp.d_o, q_pos, k_pos, w.causal, w.scale)
    assert_close(host(o), o_ref, "bf16", "o")
    assert_close(host(lse), lse_ref, "bf16", "lse", lse=True)
    assert_close(host(dq), dq_r, "bf16", "dq")
    assert_close(host(st.st_cast_from_f32(dq, st.ST_BF16)), dq_r, "bf16", "dq bf16")
    for j in range(w.n_chunks):
        assert_close(host(dk[j]), dk_r[j], "bf16", f"dk[{j}]")
        assert_close(host(dv[j]), dv_r[j], "bf16", f"dv[{j}]")
    return dq, dk, dv


@pytest.mark.parametrize("mode", [st.ST_RING_STEPWISE, st.ST_RING_FUSED], ids=["stepwise", "fused"])
@pytest.mark.parametrize("D", [128, 64])
def test_ring_fwd_bwd_small(mode, D):
    w = si.Workload("ring_bf16_small", 95, "bf16", 1, 4, 2, D, 200, 200, 8, 5 * 200, True, True)
    for C in (1, 2):
        order, members = st.st_visit_order(8, C, 5)
        print(f"[ring small D={D}] mode {mode} C={C}", flush=True)
        _ring_fwd_bwd(w, order, members, mode)


def test_backward_is_bit_reproducible():
    w = si.Workload("ring_bf16_repro", 96, "bf16", 1, 4, 1, 128, 300, 300, 4, 900, True, True)
    a = _ring_fwd_bwd(w, [0, 1, 2, 3], None, st.ST_RING_FUSED)
    b = _ring_fwd_bwd(w, [0, 1, 2, 3], None, st.ST_RING_FUSED)
    assert torch.equal(a[0], b[0])
    for j in range(4):
        assert torch.equal(a[1][j], b[1][j]) and torch.equal(a[2][j], b[2][j])
    # another visit order changes the forward's rounding (hence lse and Delta), so the gradients
    # agree with the oracle (checked inside the helper) but not bit for bit
    _ring_fwd_bwd(w, [3, 1, 0, 2], [0, 1, 0, 1], st.ST_RING_FUSED)


@pytest.mark.parametrize("D", [128, 64])
def test_dkv_tiles_through_the_queue(D):
    """513 full key tiles (57 chunks x 9 KV heads, one 256-key tile each): at two tiles per CU and more the fused
    dK/dV launch keeps one workgroup per CU and hands the tiles out through per-XCD counters; 513 is not a
    multiple of 8, so the last XCD's range is short and its workgroups take tiles of the others.  Which workgroup
    computes a tile does not change its arithmetic: two runs, and a run without the queue, agree bit for bit."""
    n = 57
    w = si.Workload(f"dkv_queue_d{D}", 99, "bf16", 1, 9, 9, D, 96, 256, n, n * 256 - 96, True, True)
    order = list(range(n - 1, -1, -1))
    print(f"[dkv queue D={D}] {n} chunks x 9 heads", flush=True)
    a = _ring_fwd_bwd(w, order, None, st.ST_RING_FUSED)
    b = _ring_fwd_bwd(w, order, None, st.ST_RING_FUSED)
    with launcher_switch("dkv_queue", 0, 1):         # every tile a workgroup of its own
        c = _ring_fwd_bwd(w, order, None, st.ST_RING_FUSED)
    for j in range(n):
        assert torch.equal(a[1][j], b[1][j]) and torch.equal(a[2][j], b[2][j])
        assert torch.equal(a[1][j], c[1][j]) and torch.equal(a[2][j], c[2][j])


LAST_CASES = [
    # three chunks the fast dK/dV kernel alone writes (it assigns and casts them itself) and the diagonal one,
    # which is zeroed, added to and cast by launches of their own
    si.Workload("last_mixed_d128", 101, "bf16", 1, 4, 2, 128, 96, 512, 4, 4 * 512 - 96, True, True),
    si.Workload("last_mixed_d64", 102, "bf16", 2, 4, 4, 64, 64, 256, 3, 3 * 256 - 64, True, True),
    # no chunk qualifies (ragged sizes): everything through the fill / add / cast launches
    si.Workload("last_ragged_d128", 103, "bf16", 1, 2, 1, 128, 100, 300, 3, 2 * 300, True, True),
    # full mask, 520 key tiles: the fast kernel's queue path with the assigning, casting epilogue
    si.Workload("last_queue_d128", 104, "bf16", 1, 8, 8, 128, 64, 256, 65, 0, False, True),
]


@pytest.mark.parametrize("w", LAST_CASES, ids=[w.name for w in LAST_CASES])
def test_ring_bwd_last_visit(w):
    """st_ring_bwd_last against st_ring_bwd: assigning into accumulators full of NaN gives, bit for bit, what adding
    into zeroed ones gives; the bf16 copies are the rounded accumulators; adding (no assign) with copies gives
    start + contribution; a listed chunk in the causal future is set to zero."""
    inp = si.make_inputs(w)
    q, ks, vs, d_o = upload(inp)
    n = w.n_chunks
    koffs = [w.k_offset(j) for j in range(n)]
    order = list(range(n))
    o, lse, o_low = st.st_ring_fwd(q, ks, vs, w.q_offset, koffs, w.causal, w.scale, order, None, st.ST_RING_FUSED)
    zeros = lambda: [torch.zeros(k.shape, device="cuda") for k in ks]
    nans = lambda: [torch.full(k.shape, float("nan"), device="cuda") for k in ks]
    lows = lambda: [torch.full(k.shape, float("nan"), device="cuda", dtype=torch.bfloat16) for k in ks]
    dq0, dk0, dv0 = torch.zeros_like(o), zeros(), zeros()
    st.st_ring_bwd(q, ks, vs, d_o, o_low, lse, w.q_offset, koffs, w.causal, w.scale, order, dq0, dk0, dv0)
    q_pos, k_pos = positions(w)
    _, dk_r, dv_r = oa.attention_backward(inp.q, inp.k, inp.v, inp.d_o, q_pos, k_pos, w.causal, w.scale)
    for j in range(n):
        assert_close(host(dk0[j]), dk_r[j], "bf16", f"dk[{j}]")
        assert_close(host(dv0[j]), dv_r[j], "bf16", f"dv[{j}]")
    for mode in (st.ST_RING_FUSED, st.ST_RING_STEPWISE):
        print(f"[{w.name}] assign + copies, mode {mode}", flush=True)
        dq1, dk1, dv1, lk1, lv1 = torch.zeros_like(o), nans(), nans(), lows(), lows()
        st.st_ring_bwd_last(q, ks, vs, d_o, o_low, lse, w.q_offset, koffs, w.causal, w.scale, order, dq1, dk1, dv1,
                            assign=True, dk_lowp=lk1, dv_lowp=lv1, mode=mode)
        if mode == st.ST_RING_FUSED:                 # step by step dq is added up in another order
            assert torch.equal(dq0, dq1)
        for j in range(n):
            assert torch.equal(dk0[j], dk1[j]) and torch.equal(dv0[j], dv1[j]), f"chunk {j}"
            assert torch.equal(lk1[j], dk1[j].to(torch.bfloat16)) and torch.equal(lv1[j], dv1[j].to(torch.bfloat16)), f"copy {j}"
    print(f"[{w.name}] assign, no copies", flush=True)
    dq2, dk2, dv2 = torch.zeros_like(o), nans(), nans()
    st.st_ring_bwd_last(q, ks, vs, d_o, o_low, lse, w.q_offset, koffs, w.causal, w.scale, order, dq2, dk2, dv2, assign=True)
    for j in range(n):
        assert torch.equal(dk0[j], dk2[j]) and torch.equal(dv0[j], dv2[j]), f"chunk {j}"
    print(f"[{w.name}] add, copies of some chunks", flush=True)
    start = [torch.randn(k.shape, device="cuda") for k in ks]
    dq3, dk3, dv3 = torch.zeros_like(o), [t.clone() for t in start], [t.clone() for t in start]
    lk3, lv3 = lows(), lows()
    some = [(lk3[j] if j % 2 == 0 else None) for j in range(n)], [(lv3[j] if j % 2 == 0 else None) for j in range(n)]
    st.st_ring_bwd_last(q, ks, vs, d_o, o_low, lse, w.q_offset, koffs, w.causal, w.scale, order, dq3, dk3, dv3,
                        assign=False, dk_lowp=some[0], dv_lowp=some[1])
    for j in range(n):
        assert_close(host(dk3[j]) - host(start[j]), dk_r[j], "bf16", f"dk[{j}] - start")
        assert_close(host(dv3[j]) - host(start[j]), dv_r[j], "bf16", f"dv[{j}] - start")
        if j % 2 == 0:
            assert torch.equal(lk3[j], dk3[j].to(torch.bfloat16)) and torch.equal(lv3[j], dv3[j].to(torch.bfloat16))
        else:
            assert torch.isnan(lk3[j].float()).all()          # not asked for: untouched
    if w.causal:
        print(f"[{w.name}] a listed chunk in the causal future", flush=True)
        koffs_f = koffs[:-1] + [w.q_offset + w.Sq + 5]          # the last chunk now starts after the last query
        dq4, dk4, dv4, lk4, lv4 = torch.zeros_like(o), nans(), nans(), lows(), lows()
        o4, lse4, o_low4 = st.st_ring_fwd(q, ks, vs, w.q_offset, koffs_f, w.causal, w.scale, order, None, st.ST_RING_FUSED)
        st.st_ring_bwd_last(q, ks, vs, d_o, o_low4, lse4, w.q_offset, koffs_f, w.causal, w.scale, order, dq4, dk4, dv4,
                            assign=True, dk_lowp=lk4, dv_lowp=lv4)
        assert not dk4[-1].any() and not dv4[-1].any() and not lk4[-1].any() and not lv4[-1].any()
        assert not torch.isnan(dk4[0]).any() and not torch.isnan(lk4[0].float()).any()


BHSD_CASES = [
    # a chunk table of the maximum length (64 entries) of 64-key chunks: forward and dQ loops
    si.Workload("fast_bhsd_64chunks", 97, "bf16", 2, 4, 2, 128, 288, 64, 64, 64 * 64 - 288, True, True),
    # 320-key chunks: the dK/dV loop as well (one full 256-key tile per chunk)
    si.Workload("fast_bhsd_dkv", 98, "bf16", 2, 4, 2, 128, 288, 320, 3, 3 * 320 - 288, True, True),
    # the same at head size 64
    si.Workload("fast64_bhsd_64chunks", 97, "bf16", 2, 4, 2, 64, 288, 64, 64, 64 * 64 - 288, True, True),
    si.Workload("fast64_bhsd_dkv", 98, "bf16", 2, 4, 2, 64, 288, 320, 3, 3 * 320 - 288, True, True),
]


@pytest.mark.parametrize("w", BHSD_CASES, ids=[w.name for w in BHSD_CASES])
def test_fast_kernels_strided_layout(w):
    """[B, heads, S, D] memory behind the same logical views, batch 2, GQA: the hand-scheduled kernels take
    their strides and chunk pointers from the caller, so the results must be bit-identical to the
    dense-layout run and match the oracle."""
    inp = si.make_inputs(w)
    q, ks, vs, d_o = upload(inp)
    q_pos, k_pos = positions(w)
    koffs = [w.k_offset(j) for j in range(w.n_chunks)]
    order = list(range(w.n_chunks - 1, -1, -1))

    def bhsd(t):
        return t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)      # same values, [B,H,S,D] memory

    def run(q_, ks_, vs_, do_):
        o, lse, o_low = st.st_ring_fwd(q_, ks_, vs_, w.q_offset, koffs, w.causal, w.scale, order, None, st.ST_RING_FUSED)
        dq = torch.zeros_like(o)
        dk = [torch.zeros(k.shape, device="cuda") for k in ks]
        dv = [torch.zeros(k.shape, device="cuda") for k in ks]
        st.st_ring_bwd(q_, ks_, vs_, do_, o_low, lse, w.q_offset, koffs, w.causal, w.scale, order, dq, dk, dv,
                       st.ST_RING_FUSED)
        torch.cuda.synchronize()
        return o, lse, dq, dk, dv

    a = run(q, ks, vs, d_o)
    b = run(bhsd(q), [bhsd(k) for k in ks], [bhsd(v) for v in vs], bhsd(d_o))
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]) and torch.equal(a[2], b[2])
    for j in range(w.n_chunks):
        assert torch.equal(a[3][j], b[3][j]) and torch.equal(a[4][j], b[4][j])
    o_ref, lse_ref = oa.attention_forward(inp.q, inp.k, inp.v, q_pos, k_pos, w.causal, w.scale)
    dq_r, dk_r, dv_r = oa.attention_backward(inp.q, inp.k, inp.v, inp.d_o, q_pos, k_pos, w.causal, w.scale)
    assert_close(host(a[0]), o_ref, "bf16", "o")
    assert_close(host(a[1]), lse_ref, "bf16", "lse", lse=True)
    assert_close(host(a[2]), dq_r, "bf16", "dq")
    for j in range(w.n_chunks):
        assert_close(host(a[3][j]), dk_r[j], "bf16", f"dk[{j}]")
        assert_close(host(a[4][j]), dv_r[j], "bf16", f"dv[{j}]")


def test_degenerate_shapes():
    """Nothing to do is legal everywhere: no query rows, batch 0, an empty visit list, zero elements to cast."""
    dev = "cuda"
    for B, Sq in ((1, 0), (0, 64)):
        q = torch.zeros((B, Sq, 2, 128), dtype=torch.bfloat16, device=dev)
        k = torch.zeros((B, 64, 1, 128), dtype=torch.bfloat16, device=dev)
        o, lse = st.st_attn_block_fwd(q, k, k, 0, 0, True, 0.1)
        assert o.shape == (B, Sq, 2, 128) and lse.shape == (B, 2, Sq)
        o, lse, low = st.st_ring_fwd(q, [k], [k], 0, [0], True, 0.1, [0])
        delta = st.st_attn_delta(q, o)
        dq = torch.zeros_like(o)
        dk, dv = torch.zeros(k.shape, device=dev), torch.zeros(k.shape, device=dev)
        st.st_attn_block_bwd(q, k, k, q, lse, delta, 0, 0, True, 0.1, dq, dk, dv)
        st.st_ring_bwd(q, [k], [k], q, low, lse, 0, [0], True, 0.1, [0], dq, [dk], [dv])
        st.st_attn_merge(o, lse, torch.zeros_like(o), torch.zeros_like(lse))
        oc, lc = st.st_attn_combine([o, o.clone()], [lse, lse.clone()])
        assert oc.shape == o.shape and lc.shape == lse.shape
        assert st.st_cast_from_f32(o, st.ST_BF16).shape == o.shape
        torch.cuda.synchronize()
        assert not dk.any() and not dv.any()
    # an empty visit list: the state is the empty state, the gradients stay as they were
    q = torch.randn((1, 40, 2, 128), device=dev).to(torch.bfloat16)
    k = torch.randn((1, 64, 1, 128), device=dev).to(torch.bfloat16)
    o, lse, low = st.st_ring_fwd(q, [k], [k], 0, [0], False, 0.1, [])
    dq = torch.ones((1, 40, 2, 128), device=dev)
    dk, dv = torch.ones(k.shape, device=dev), torch.ones(k.shape, device=dev)
    st.st_ring_bwd(q, [k], [k], q, low, lse, 0, [0], False, 0.1, [], dq, [dk], [dv])
    torch.cuda.synchronize()
    assert not o.any() and torch.isneginf(lse).all() and not low.any()
    assert bool((dq == 1).all()) and bool((dk == 1).all()) and bool((dv == 1).all())


# ---- peaked softmax: a wide spread of the scores -------------------------------------------------------------
# Later K chunks are scaled up (k_ramp), or Q, K, V and dO all carry a larger sigma, so that the scores of a row
# spread over 10 log2 units and more and a few keys carry nearly all of its probability.  The gradients are then
# far larger than 1 (max |dQ| about 10 to 20), where the benchmark's absolute bound of 2e-2, stated for unit-scale
# data, is below the bf16 rounding of P and dS themselves (2^-9 relative): see assert_close_wide for the bound used.
WIDE_CASES = [
    # name, Hq, Hkv, Sq, Sk, n, causal, k_ramp, sigma
    ("ramp_causal_gqa", 4, 2, 512, 512, 4, True, 0.5, 1.0),
    ("ramp_full_mask", 2, 2, 256, 256, 6, False, 0.5, 1.0),
    ("sigma2_causal", 2, 1, 512, 256, 4, True, 0.0, 2.0),
]


@pytest.mark.parametrize("mode", [st.ST_RING_STEPWISE, st.ST_RING_FUSED], ids=["stepwise", "fused"])
@pytest.mark.parametrize("D", [128, 64])
@pytest.mark.parametrize("case", WIDE_CASES, ids=[c[0] for c in WIDE_CASES])
def test_backward_at_a_wide_score_spread(case, D, mode):
    name, Hq, Hkv, Sq, Sk, n, causal, k_ramp, sigma = case
    w = si.Workload(f"wide_{name}_d{D}", 97, "bf16", 1, Hq, Hkv, D, Sq, Sk, n, n * Sk - Sq if causal else 0, causal, True,
                    sigma=sigma, k_ramp=k_ramp)
    inp = si.make_inputs(w)
    q, ks, vs, d_o = upload(inp)
    q_pos, k_pos = positions(w)
    koffs = [w.k_offset(j) for j in range(w.n_chunks)]
    order = list(range(n - 1, -1, -1))
    print(f"[{w.name}] mode {mode}", flush=True)
    o, lse, o_low = st.st_ring_fwd(q, ks, vs, w.q_offset, koffs, w.causal, w.scale, order, None, mode)
    dq = torch.zeros_like(o)
    dk = [torch.zeros(k.shape, device="cuda") for k in ks]
    dv = [torch.zeros(k.shape, device="cuda") for k in ks]
    st.st_ring_bwd(q, ks, vs, d_o, o_low, lse, w.q_offset, koffs, w.causal, w.scale, order, dq, dk, dv, mode)
    torch.cuda.synchronize()
    o_ref, lse_ref = oa.attention_forward(inp.q, inp.k, inp.v, q_pos, k_pos, w.causal, w.scale)
    dq_r, dk_r, dv_r = oa.attention_backward(inp.q, inp.k, inp.v, inp.d_o, q_pos, k_pos, w.causal, w.scale)
    # the spread this case is about: standard deviation of a row's visible scores, in log2 units
    s0 = (inp.q[0, :, 0].astype(np.float64) @ inp.k[-1][0, :, 0].astype(np.float64).T) * w.scale * np.log2(np.e)
    assert s0.std() > 2.0, f"scores spread over only {s0.std():.2f} log2 units"
    report = {"o": assert_close_wide(host(o), o_ref, "o"), "dq": assert_close_wide(host(dq), dq_r, "dq"),
              "lse": assert_close_wide(host(lse), lse_ref, "lse", lse=True)}
    report["dk"] = assert_close_wide(torch.cat([host_t(x) for x in dk], 1), np.concatenate(dk_r, 1), "dk")
    report["dv"] = assert_close_wide(torch.cat([host_t(x) for x in dv], 1), np.concatenate(dv_r, 1), "dv")
    print(f"[{w.name}] " + ", ".join(f"{k}: max/top {v[0]:.2e} fro {v[1]:.2e}" for k, v in report.items()), flush=True)


def host_t(t):
    return t.detach().double().cpu()
