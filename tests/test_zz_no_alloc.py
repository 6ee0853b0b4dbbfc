"""GPU test of st_ring_bwd_noalloc, the entry point that works on the library's static scratch: its results equal
those of st_ring_bwd (same kernels, the workspace being the only difference) bit for bit, on two calls in a
row, the second with a smaller input; a share beyond the scratch is refused before anything is enqueued."""
import numpy as np
import pytest
import torch

import paper_2407_00611_amd as st
import synth_inputs as si
from oracle import attention as oa
from util import assert_close, host, positions, upload

pytestmark = pytest.mark.gpu


def _both_ways(w, order, mode):
    inp = si.make_inputs(w)
    q, ks, vs, d_o = upload(inp)
    koffs = [w.k_offset(j) for j in range(w.n_chunks)]
    o, lse, o_low = st.st_ring_fwd(q, ks, vs, w.q_offset, koffs, w.causal, w.scale, order, None, mode)
    out = []
    for entry in (st.st_ring_bwd, st.st_ring_bwd_noalloc):
        dq = torch.zeros_like(o)
        dk = [torch.zeros(k.shape, device="cuda") for k in ks]
        dv = [torch.zeros(k.shape, device="cuda") for k in ks]
        print(f"[{w.name}] {entry.__name__} mode {mode}", flush=True)
        entry(q, ks, vs, d_o, o_low, lse, w.q_offset, koffs, w.causal, w.scale, order, dq, dk, dv, mode)
        torch.cuda.synchronize()
        out.append((dq, dk, dv))
    (dq_a, dk_a, dv_a), (dq_b, dk_b, dv_b) = out
    assert torch.equal(dq_a, dq_b), "dq differs from st_ring_bwd"
    for j in range(w.n_chunks):
        assert torch.equal(dk_a[j], dk_b[j]) and torch.equal(dv_a[j], dv_b[j]), f"chunk {j} differs from st_ring_bwd"
    # and both are right
    q_pos, k_pos = positions(w)
    dq_r, dk_r, dv_r = oa.attention_backward(inp.q, inp.k, inp.v, inp.d_o, q_pos, k_pos, w.causal, w.scale)
    dt = "bf16" if w.dtype == "bf16" else "f32"
    assert_close(host(dq_b), dq_r, dt, "dq")
    for j in range(w.n_chunks):
        assert_close(host(dk_b[j]), dk_r[j], dt, f"dk[{j}]")
        assert_close(host(dv_b[j]), dv_r[j], dt, f"dv[{j}]")


@pytest.mark.parametrize("mode", [st.ST_RING_FUSED, st.ST_RING_STEPWISE], ids=["fused", "stepwise"])
def test_static_scratch_matches_workspace_on_two_calls_in_a_row(mode):
    # first the larger share (hand-scheduled kernels, tile queue, ragged rows), then a smaller one that leaves
    # most of what the first call wrote into the scratch in place
    big = si.Workload("noalloc_big", 111, "bf16", 1, 4, 2, 128, 600, 512, 5, 5 * 512 - 600, True, True)
    small = si.Workload("noalloc_small", 112, "bf16", 1, 2, 1, 64, 96, 256, 2, 2 * 256 - 96, True, True)
    _both_ways(big, [4, 0, 2, 1, 3], mode)
    _both_ways(small, [1, 0], mode)
    tiny = si.Workload("noalloc_f32", 113, "f32", 1, 2, 1, 64, 40, 48, 2, 56, True, True)
    _both_ways(tiny, [0, 1], mode)


def test_a_share_beyond_the_scratch_is_refused():
    limit = st.st_ring_bwd_noalloc_max_bytes()
    assert limit == 40 << 20
    B, Sq, Hq, Hkv, D, Sk = 1, 8192, 32, 8, 128, 256          # Q' alone is 64 MiB
    q = torch.zeros((B, Sq, Hq, D), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((B, Sk, Hkv, D), dtype=torch.bfloat16, device="cuda")
    assert st.st_ring_workspace_bytes(q, [k], [k], 0, [0], True, 0.1, st.ST_RING_FUSED, True) > limit
    lse = torch.zeros((B, Hq, Sq), device="cuda")
    dq = torch.full((B, Sq, Hq, D), 7.0, device="cuda")
    dk = [torch.full(k.shape, 7.0, device="cuda")]
    dv = [torch.full(k.shape, 7.0, device="cuda")]
    with pytest.raises(st.StarTrailError) as e:
        st.st_ring_bwd_noalloc(q, [k], [k], q, q, lse, 0, [0], True, 0.1, [0], dq, dk, dv)
    assert e.value.status == 5 and "static scratch" in str(e.value)
    torch.cuda.synchronize()
    assert float(dq.min()) == 7.0 and float(dk[0].min()) == 7.0 and float(dv[0].min()) == 7.0   # nothing ran
