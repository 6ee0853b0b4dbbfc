"""GPU parity, bf16 forward (MFMA path) against the fp64 oracle on the bf16-rounded inputs.
Tolerance: max abs 2e-2 and relative Frobenius 1e-2 (lse: max abs 2e-2)."""
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
    # full 256-query tiles: the hand-scheduled loop takes the fully visible 64-key tiles, the general kernel the rest
    ("fast_one_tile", 1, 1, 1, 128, 256, 64, 1, 0, False),
    ("fast_two_tiles", 1, 1, 1, 128, 256, 128, 1, 0, False),
    ("fast_chunk_switches", 2, 4, 2, 128, 300, 320, 3, 0, False),
    ("fast_causal_mix", 1, 2, 1, 128, 512, 200, 5, 520, True),
    # the same loop generated for head size 64
    ("fast64_one_tile", 1, 1, 1, 64, 256, 64, 1, 0, False),
    ("fast64_two_tiles", 1, 1, 1, 64, 256, 128, 1, 0, False),
    ("fast64_chunk_switches", 2, 4, 2, 64, 300, 320, 3, 0, False),
    ("fast64_causal_mix", 1, 2, 1, 64, 512, 200, 5, 520, True),
    ("fast64_long", 1, 3, 3, 64, 256, 1024, 3, 0, False),
]


def _workload(c):
    name, B, Hq, Hkv, D, Sq, Sk, n, q0, causal = c
    return si.Workload(name, 80 + len(name), "bf16", B, Hq, Hkv, D, Sq, Sk, n, q0, causal, False)


@pytest.mark.parametrize("D", [128, 64])
def test_ring_forward_rising_maxima(D):
    """Keys grow from chunk to chunk, so the row maxima jump by far more than the lazy reference tolerates:
    the rescale routine of the hand-scheduled loop runs several times per row."""
    w = si.Workload("fast_rescale", 86, "bf16", 1, 2, 1, D, 256, 192, 5, 5 * 192 - 256, True, False, k_ramp=1.0)
    inp = si.make_inputs(w)
    q, ks, vs, _ = upload(inp)
    q_pos, k_pos = positions(w)
    koffs = [w.k_offset(j) for j in range(w.n_chunks)]
    o_ref, lse_ref = oa.attention_forward(inp.q, inp.k, inp.v, q_pos, k_pos, w.causal, w.scale)
    for order in ([0, 1, 2, 3, 4], [4, 0, 3, 1, 2]):
        print(f"[fast_rescale] order {order}", flush=True)
        o, lse, o_low = st.st_ring_fwd(q, ks, vs, w.q_offset, koffs, w.causal, w.scale, order, None, st.ST_RING_FUSED)
        # the last chunk's keys are five times the first one's: scores spread over some 7 log2 units (one sigma)
        assert_close_wide(host(o), o_ref, "o")
        assert_close_wide(host(lse), lse_ref, "lse", lse=True)
        assert_close_wide(host(o_low), o_ref, "o bf16")


@pytest.mark.parametrize("case", STEP_CASES, ids=[c[0] for c in STEP_CASES])
def test_block_fwd_then_merge(case):
    w = _workload(case)
    inp = si.make_inputs(w)
    q, ks, vs, _ = upload(inp)
    q_pos, k_pos = positions(w)
    o_acc = torch.zeros((w.B, w.Sq, w.Hq, w.D), device="cuda")
    lse_acc = torch.full((w.B, w.Hq, w.Sq), -float("inf"), device="cuda")
    for j in range(w.n_chunks):
        print(f"[{w.name}] block_fwd chunk {j}", flush=True)
        o_p, l_p = st.st_attn_block_fwd(q, ks[j], vs[j], w.q_offset, w.k_offset(j), w.causal, w.scale)
        o_pr, l_pr = oa.block_forward(inp.q, inp.k[j], inp.v[j], q_pos, k_pos[j], w.causal, w.scale)
        assert_close(host(o_p), o_pr, "bf16", f"o_part[{j}]")
        assert_close(host(l_p), l_pr, "bf16", f"lse_part[{j}]", lse=True)
        st.st_attn_merge(o_acc, lse_acc, o_p, l_p)
    o_mono, lse_mono = oa.attention_forward(inp.q, inp.k, inp.v, q_pos, k_pos, w.causal, w.scale)
    assert_close(host(o_acc), o_mono, "bf16", "o vs monolithic")
    assert_close(host(lse_acc), lse_mono, "bf16", "lse vs monolithic", lse=True)


@pytest.mark.parametrize("mode", [st.ST_RING_STEPWISE, st.ST_RING_FUSED], ids=["stepwise", "fused"])
@pytest.mark.parametrize("D", [128, 64])
def test_ring_forward_small(mode, D):
    w = si.Workload("ring_bf16_small", 85, "bf16", 1, 4, 2, D, 200, 200, 8, 5 * 200, True, False)
    inp = si.make_inputs(w)
    q, ks, vs, _ = upload(inp)
    q_pos, k_pos = positions(w)
    koffs = [w.k_offset(j) for j in range(w.n_chunks)]
    o_ref, lse_ref = oa.attention_forward(inp.q, inp.k, inp.v, q_pos, k_pos, w.causal, w.scale)
    for C in (1, 2):
        order, members = st.st_visit_order(8, C, 5)
        print(f"[ring small D={D}] mode {mode} C={C} order {order}", flush=True)
        o, lse, o_low = st.st_ring_fwd(q, ks, vs, w.q_offset, koffs, w.causal, w.scale, order, members, mode)
        assert_close(host(o), o_ref, "bf16", "o")
        assert_close(host(lse), lse_ref, "bf16", "lse", lse=True)
        assert_close(host(o_low), o_ref, "bf16", "o bf16")
        assert torch.equal(o_low, o.to(torch.bfloat16))


@pytest.mark.parametrize("mode", [st.ST_RING_STEPWISE, st.ST_RING_FUSED], ids=["stepwise", "fused"])
def test_config2_forward(mode):
    w = si.paper_workloads()[1]
    inp = si.make_inputs(w)
    q, ks, vs, _ = upload(inp)
    q_pos, k_pos = positions(w)
    koffs = [w.k_offset(j) for j in range(w.n_chunks)]
    order, members = st.st_visit_order(w.ring_P, w.ring_C, w.ring_rank)
    print(f"[cfg2] mode {mode}", flush=True)
    o, lse, o_low = st.st_ring_fwd(q, ks, vs, w.q_offset, koffs, w.causal, w.scale, order, members, mode)
    torch.cuda.synchronize()
    print("[cfg2] oracle", flush=True)
    o_ref, lse_ref = oa.attention_forward(inp.q, inp.k, inp.v, q_pos, k_pos, w.causal, w.scale)
    assert_close(host(o), o_ref, "bf16", "o")
    assert_close(host(lse), lse_ref, "bf16", "lse", lse=True)
    assert_close(host(o_low), o_ref, "bf16", "o bf16")


def test_empty_and_future_chunks():
    w = _workload(("edge", 1, 2, 1, 128, 70, 40, 1, 0, True))
    inp = si.make_inputs(w)
    q, ks, vs, _ = upload(inp)
    o, l = st.st_attn_block_fwd(q, ks[0], vs[0], 0, 1000, True, w.scale)          # chunk in the future
    assert not o.any() and torch.isneginf(l).all()
    o, l = st.st_attn_block_fwd(q, ks[0][:, :0], vs[0][:, :0], 0, 0, False, w.scale)   # Sk = 0
    assert not o.any() and torch.isneginf(l).all()
    o, l, ol = st.st_ring_fwd(q, ks, vs, 0, [1000], True, w.scale, [0])            # whole share invisible
    assert not o.any() and torch.isneginf(l).all() and not ol.any()


MANY = [
    # name, D, Sq, Sk, chunks, visited (None: all)
    ("three_launches_d128", 128, 300, 64, 150, None),
    ("subset_of_many_d128", 128, 300, 64, 150, 50),
    ("most_chunks_d64", 64, 70, 16, 256, None),
]


@pytest.mark.parametrize("case", MANY, ids=[c[0] for c in MANY])
def test_many_chunks_forward_and_backward(case):
    """More chunks than one launch's table holds (64), up to the most a call accepts (256), and a visited subset
    of a long table: the fused driver walks them in several launches, or splits one under-filled launch."""
    name, D, Sq, Sk, n, visited = case
    w = si.Workload(name, 85, "bf16", 1, 2, 1, D, Sq, Sk, n, n * Sk - Sq - 40, True, True)
    inp = si.make_inputs(w, threads=8)
    q, ks, vs, d_o = upload(inp)
    q_pos, k_pos = positions(w)
    koffs = [w.k_offset(j) for j in range(n)]
    order = list(range(n - 1, -1, -1)) if visited is None else list(range(n - 1, -1, -3))[:visited]
    sub = sorted(order)
    o_ref, lse_ref = oa.attention_forward(inp.q, [inp.k[j] for j in sub], [inp.v[j] for j in sub], q_pos,
                                          [k_pos[j] for j in sub], True, w.scale)
    dq_ref, dk_ref, dv_ref = oa.attention_backward(inp.q, [inp.k[j] for j in sub], [inp.v[j] for j in sub], inp.d_o, q_pos,
                                                   [k_pos[j] for j in sub], True, w.scale)
    o, lse, o_low = st.st_ring_fwd(q, ks, vs, w.q_offset, koffs, True, w.scale, order, None, st.ST_RING_FUSED)
    dq = torch.zeros_like(o)
    dk = [torch.zeros(k.shape, device="cuda") for k in ks]
    dv = [torch.zeros(k.shape, device="cuda") for k in ks]
    st.st_ring_bwd(q, ks, vs, d_o, o_low, lse, w.q_offset, koffs, True, w.scale, order, dq, dk, dv, st.ST_RING_FUSED)
    torch.cuda.synchronize()
    assert_close(host(o), o_ref, "bf16", "o")
    assert_close(host(lse), lse_ref, "bf16", "lse", lse=True)
    assert torch.equal(o_low, o.to(torch.bfloat16))
    assert_close(host(dq), dq_ref, "bf16", "dq")
    for x, j in enumerate(sub):
        assert_close(host(dk[j]), dk_ref[x], "bf16", f"dk {j}")
        assert_close(host(dv[j]), dv_ref[x], "bf16", f"dv {j}")
    for j in set(range(n)) - set(sub):
        assert float(dk[j].abs().max()) == 0.0 and float(dv[j].abs().max()) == 0.0


@pytest.mark.parametrize("gap", ["0", "0.5", "2"])
@pytest.mark.parametrize("D", [128, 64])
def test_forward_with_a_tight_exponent_reference(D, gap):
    """The launcher switch "fwd_gap" (a testing override of the hand-scheduled loop) lets a block maximum exceed
    the lazy exponent reference by only `gap` log2 units, so the rescale routine runs in most blocks of the walk
    (both score buffers, the last tile's blocks, several times per row) instead of a few times per kernel."""
    with launcher_switch("fwd_gap", float(gap), 8.0):
        _tight_reference_case(D, gap)


def _tight_reference_case(D, gap):
    w = si.Workload("fast_tight_reference", 87, "bf16", 1, 2, 1, D, 512, 192, 6, 6 * 192 - 512, True, False, k_ramp=0.4)
    inp = si.make_inputs(w)
    q, ks, vs, _ = upload(inp)
    q_pos, k_pos = positions(w)
    koffs = [w.k_offset(j) for j in range(w.n_chunks)]
    o_ref, lse_ref = oa.attention_forward(inp.q, inp.k, inp.v, q_pos, k_pos, w.causal, w.scale)
    for order in ([0, 1, 2, 3, 4, 5], [5, 2, 0, 4, 1, 3], [3]):
        sub = sorted(order)
        if len(order) < w.n_chunks:
            o_r, l_r = oa.attention_forward(inp.q, [inp.k[j] for j in sub], [inp.v[j] for j in sub], q_pos,
                                            [k_pos[j] for j in sub], w.causal, w.scale)
        else:
            o_r, l_r = o_ref, lse_ref
        o, lse, o_low = st.st_ring_fwd(q, ks, vs, w.q_offset, koffs, w.causal, w.scale, order, None, st.ST_RING_FUSED)
        torch.cuda.synchronize()
        assert_close(host(o), o_r, "bf16", f"o, order {order}")
        assert_close(host(lse), l_r, "bf16", f"lse, order {order}", lse=True)


@pytest.mark.parametrize("D", [128, 64])
@pytest.mark.parametrize("Sq,causal", [(512, True), (300, True), (600, False), (256, True)])
def test_split_forward_on_a_poisoned_workspace(D, Sq, causal):
    """Under-filled fused forward: the query tiles are split over the chunks, hand-scheduled and general
    workgroups run side by side in one launch and the partial states (one per split, one for the masked and
    ragged tiles) are combined.  The workspace starts out full of NaN, so a state row nobody wrote, or one that
    is read although it is empty, shows; ragged row counts leave rows that only the general workgroups cover."""
    n, Sk = 7, 320
    w = si.Workload(f"split_sq{Sq}", 88, "bf16", 1, 2, 1, D, Sq, Sk, n, (n - 2) * Sk - Sq + 100 if causal else 0, causal, False)
    inp = si.make_inputs(w)
    q, ks, vs, _ = upload(inp)
    q_pos, k_pos = positions(w)
    koffs = [w.k_offset(j) for j in range(n)]
    need = st.st_ring_workspace_bytes(q, ks, vs, w.q_offset, koffs, w.causal, w.scale, st.ST_RING_FUSED, False)
    assert need >= 3 * q.numel() * 4, "this shape is meant to take the split path"
    for order in (list(range(n)), [5, 1, 3], [6, 4]):
        ws = torch.full((need + 256,), 0xFF, dtype=torch.uint8, device="cuda")
        print(f"[{w.name} D={D}] order {order}", flush=True)
        o, lse, o_low = st.st_ring_fwd(q, ks, vs, w.q_offset, koffs, w.causal, w.scale, order, None, st.ST_RING_FUSED,
                                       workspace=ws)
        torch.cuda.synchronize()
        sub = sorted(order)
        o_r, l_r = oa.attention_forward(inp.q, [inp.k[j] for j in sub], [inp.v[j] for j in sub], q_pos,
                                        [k_pos[j] for j in sub], w.causal, w.scale)
        assert_close(host(o), o_r, "bf16", f"o, order {order}")
        assert_close(host(lse), l_r, "bf16", f"lse, order {order}", lse=True)
        assert torch.equal(o_low, o.to(torch.bfloat16))


def test_split_forward_replayed_from_a_hip_graph():
    """The launch-bound forward of the benchmark's second configuration is timed as a HIP graph replay.  The
    library only enqueues kernels (no memset nodes), so the captured graph is the whole call: every replay, with
    eager calls and synchronisations between them, gives the eager result bit for bit."""
    w = si.Workload("graph_split", 89, "bf16", 1, 4, 4, 128, 512, 256, 6, 4 * 256 - 100, True, False)
    inp = si.make_inputs(w)
    q, ks, vs, _ = upload(inp)
    koffs = [w.k_offset(j) for j in range(w.n_chunks)]
    order = [0, 1, 2, 3, 4, 5]
    need = st.st_ring_workspace_bytes(q, ks, vs, w.q_offset, koffs, w.causal, w.scale, st.ST_RING_FUSED, False)
    ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
    o = torch.empty((w.B, w.Sq, w.Hq, w.D), device="cuda")
    lse = torch.empty((w.B, w.Hq, w.Sq), device="cuda")
    low = torch.empty((w.B, w.Sq, w.Hq, w.D), dtype=torch.bfloat16, device="cuda")

    def call():
        st.st_ring_fwd(q, ks, vs, w.q_offset, koffs, w.causal, w.scale, order, None, st.ST_RING_FUSED,
                       o_acc=o, lse=lse, o_lowp=low, workspace=ws)

    call()
    torch.cuda.synchronize()
    ref = (o.clone(), lse.clone(), low.clone())
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for rep in range(4):
        print(f"[graph_split] replay {rep}", flush=True)
        o.fill_(float("nan")); lse.fill_(float("nan")); low.fill_(float("nan")); ws.fill_(0xFF)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o, ref[0]) and torch.equal(lse, ref[1]) and torch.equal(low, ref[2]), f"replay {rep}"
        # eager work of the same kind between the replays
        o.zero_()
        call()
        torch.cuda.synchronize()
        assert torch.equal(o, ref[0])
