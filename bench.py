#!/usr/bin/env python3
"""Benchmark: one GPU's share of ring attention, forward + backward, on one MI355X.

A step = one pass of the whole hot path over the workload, with all inputs resident in HBM:
  visit order -> ring forward (all chunks, online-softmax state, O in fp32 and bf16, lse)
  -> zero the dQ accumulator -> Delta -> ring backward (dK/dV and dQ kernels; this visit being the chunks' only
  one, dK / dV are assigned in fp32 and rounded to bf16 by the kernels that produce them) -> fp32 -> bf16 cast of dQ.
The workload is benchmark configuration 4 (GQA 32/8 heads, D=128, Q shard 4096, 32 chunks of
4096 keys, causal, last rank of a P=32 / C=4 concentric layout) with synthetic N(0,1) bf16 data.

`--shape team` times the same model in the shape one GPU of the concentric layout really sees (the team's
gathered 16384 queries against the two gathered team buffers this GPU meets, then the 4-way combine that
keeps its own 4096 rows; backward of the same shape); `--shape dit` times a ring share shaped like the
paper's diffusion-transformer runs (24 heads of size 64, full mask, 16384-token shard of 131072 tokens);
`--shape zigzag [--rank r]` times the model of configuration 4 under the load-balanced causal placement (rank
r holds pieces r and 63 - r of the sequence cut in 64);
the default `--shape ring` is the headline workload.

Prints ONE JSON line (see the keys below).  `value` is algorithmic attention TFLOP/s: 4*D per
visible (query, key) pair forward and 10*D backward, masked pairs and recomputation earn nothing.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6     # MI355X dense bf16 MFMA: 256 CU x 4096 flop/clk/CU x 2.4 GHz
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E


def hbm_traffic(kernel: str, workload: str):
    """(HBM bytes per launch of `kernel`, file they come from): counters cannot be read from inside this run, so
    the figure is the one in the committed rocprofv3 counter summary of the same kernel and workload, if any."""
    name = f"{kernel}_{workload.split('_')[0]}_hbm_traffic.txt"
    try:
        for line in open(os.path.join(ROOT, "profiles", name)):
            if line.startswith("traffic_bytes_per_launch"):
                return int(line.split("=")[1]), f"profiles/{name}"
    except OSError:
        pass
    return None, None


def mfma_ceiling(st, torch, data) -> dict:
    """What the matrix units sustain with nothing else running (st_mfma_probe: a loop of v_mfma_f32_32x32x16_bf16
    only, one workgroup per compute unit), on all-ones operands and on the workload's own Q values: the rate
    depends on the data because the chip runs at its power limit.  Median of 5 launches of about 10 ms each."""
    facts = st.st_device_facts()
    sink = torch.empty(facts["compute_units"] * 256, dtype=torch.float32, device="cuda")
    ones = torch.ones(1 << 20, dtype=torch.bfloat16, device="cuda")

    def rate(ops, mix):
        per_iter = st.st_mfma_probe(ops, 1, sink, mix)               # flop of one iteration
        iters = max(1, int(1.9e13 / per_iter))                        # about 10 ms
        st.st_mfma_probe(ops, max(1, iters // 100), sink, mix)
        ms = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            flop = st.st_mfma_probe(ops, iters, sink, mix)
            e1.record()
            torch.cuda.synchronize()
            ms.append(e0.elapsed_time(e1))
        return round(flop / (sorted(ms)[2] * 1e-3) / 1e12, 1)

    out = {"ones": rate(ones, 0), "workload_q": rate(data.reshape(-1), 0)}
    # the same loop with side instructions beside the MFMAs, on the workload's data: the price of each kind of
    # instruction, and the ceiling of each hand-scheduled loop's instruction mix (head size 128)
    out["workload_q_with_side_instructions"] = {
        st.st_mfma_probe_mix_name(m): rate(data.reshape(-1), m) for m in range(1, st.st_mfma_probe_mixes() + 1)}
    return out


def queue_filler(st, torch):
    """Keeps the GPU busy for a few milliseconds (the MFMA probe on a small buffer) so that the short launches
    enqueued behind it are all in the queue before the first of them starts: their HIP-event intervals then
    measure the kernels back to back and not how fast the host can launch."""
    facts = st.st_device_facts()
    sink = torch.empty(facts["compute_units"] * 256, dtype=torch.float32, device="cuda")
    ones = torch.ones(1 << 16, dtype=torch.bfloat16, device="cuda")
    return lambda: st.st_mfma_probe(ones, 8000, sink)


def batch_time(torch, fill_queue, launch, n: int = 16, batches: int = 5) -> float:
    """Milliseconds per launch of a short kernel: n launches between two HIP events on the launch stream, enqueued
    behind a filler so that they run back to back; median of `batches` such batches."""
    per_launch = []
    for _ in range(batches):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        fill_queue()
        e0.record()
        for i in range(n):
            launch(i)
        e1.record()
        torch.cuda.synchronize()
        per_launch.append(e0.elapsed_time(e1) / n)
    return sorted(per_launch)[batches // 2]


def merge_pass(st, torch, w) -> dict:
    """HBM rate of the log-sum-exp merge (st_attn_merge) at this workload's state size.  Four buffer sets are
    rotated so that no operand of a launch is left in the 256 MB last-level cache by the launch before."""
    fill_queue = queue_filler(st, torch)
    sets = []
    for _ in range(4):
        o_a = torch.randn((w.B, w.Sq, w.Hq, w.D), device="cuda")
        o_p = torch.randn_like(o_a)
        l_a = torch.randn((w.B, w.Hq, w.Sq), device="cuda")
        l_p = torch.randn_like(l_a)
        sets.append((o_a, l_a, o_p, l_p))
    for i in range(4):
        st.st_attn_merge(*sets[i])
    ms = batch_time(torch, fill_queue, lambda i: st.st_attn_merge(*sets[i % 4]))
    rows = w.B * w.Hq * w.Sq
    nbytes = rows * (12 * w.D + 12)               # two states read, one written: D + 1 floats each
    gbs = nbytes / (ms * 1e-3) / 1e9
    return {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4),
            "bytes_per_launch": nbytes, "median_ms": round(ms, 4)}


def combine_pass(st, torch, states_o, states_l, n_own, w) -> dict:
    """HBM rate of the n-way combine (st_attn_combine) as the team-gathered step runs it: C states of the
    team's rows are read on the kept rows only, one state of n_own rows is written (fp32 and bf16).  The
    member whose rows are kept rotates, so that a launch finds none of its operands in the last-level cache
    (C x n_own rows x (4 D + 4) bytes per member, C members)."""
    Ct = len(states_o)
    o = torch.empty((w.B, n_own, w.Hq, w.D), dtype=torch.float32, device="cuda")
    l = torch.empty((w.B, w.Hq, n_own), dtype=torch.float32, device="cuda")
    low = torch.empty((w.B, n_own, w.Hq, w.D), dtype=torch.bfloat16, device="cuda")
    for a in range(Ct):
        st.st_attn_combine(states_o, states_l, a * n_own, n_own, st.ST_BF16, o_out=o, lse_out=l, o_out_lowp=low)
    ms = batch_time(torch, queue_filler(st, torch),
                    lambda i: st.st_attn_combine(states_o, states_l, (i % Ct) * n_own, n_own, st.ST_BF16, o_out=o, lse_out=l,
                                                 o_out_lowp=low))
    rows = w.B * w.Hq * n_own
    nbytes = rows * (Ct * (4 * w.D + 4) + 4 * w.D + 4 + 2 * w.D)
    gbs = nbytes / (ms * 1e-3) / 1e9
    return {"kernel": "combine", "states": Ct, "bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": round(gbs / PEAK_HBM_GBS, 4), "bytes_per_launch": nbytes, "median_ms": round(ms, 4)}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="benchmark configuration 1..5 (default 4)")
    ap.add_argument("--mode", choices=["fused", "stepwise"], default="fused")
    ap.add_argument("--shape", choices=["ring", "team", "dit", "zigzag"], default="ring",
                    help="ring: a resident N/P-row shard meets every chunk (configurations 1..5); "
                         "team: the team-gathered shape of the concentric layout (model of configuration 4); "
                         "dit: a ring share shaped like the paper's diffusion-transformer runs (24 heads x 64, full mask); "
                         "zigzag: the model of configuration 4 under the load-balanced causal placement (--rank picks the rank)")
    ap.add_argument("--rank", type=int, default=0, help="rank of the ring for --shape zigzag (0..31)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", choices=["auto", "on", "off"], default="auto",
                    help="replay the step from a HIP graph instead of launching its kernels one by one; auto: only for "
                         "launch-bound workloads (less than 0.1 TFLOP per step: configurations 1 and 2)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures ONE GPU's share of the ring; runs with more than one GPU are not part of "
              "this build (the ring is simulated over chunks resident in HBM). Use --gpus 1.", file=sys.stderr)
        return 2

    import torch

    import paper_2407_00611_amd as st
    import synth_inputs as si

    if not torch.cuda.is_available():
        print("bench.py needs a GPU (there is no CPU fallback for the HIP path)", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    team = args.shape == "team"
    w = si.team_workload() if team else si.dit_workload() if args.shape == "dit" else si.zigzag_workload(args.rank) if args.shape == "zigzag" \
        else si.paper_workloads()[args.config - 1]
    mode = st.ST_RING_FUSED if args.mode == "fused" else st.ST_RING_STEPWISE
    bf16 = w.dtype == "bf16"
    storage = st.ST_BF16 if bf16 else st.ST_F32

    # ---- inputs: generated on the host from the seeded generator, uploaded once -------------------
    t0 = time.time()
    inp = si.make_inputs(w, threads=min(16, os.cpu_count() or 8), keep_f32=not bf16)

    def up(bits, f32):
        if bf16:
            return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(f32).cuda()

    q = up(inp.q_bits, inp.q)
    ks = [up(inp.k_bits[j] if bf16 else None, inp.k[j]) for j in range(w.n_chunks)]
    vs = [up(inp.v_bits[j] if bf16 else None, inp.v[j]) for j in range(w.n_chunks)]
    d_o = up(inp.d_o_bits, inp.d_o) if w.backward else None
    koffs = [w.k_offset(j) for j in range(w.n_chunks)]
    if team:
        order, members = st.st_team_visit_order(w.ring_P, w.ring_C, w.ring_rank), None
    elif w.q_seg:
        # rank r holds pieces r and 2 P - 1 - r; the ring delivers rank (r - i) mod P's two pieces at step i
        ranks = st.st_visit_order(w.ring_P, 1, w.ring_rank)[0]
        order, members = [c for x in ranks for c in (x, 2 * w.ring_P - 1 - x)], None
    elif w.ring_P:
        order, members = st.st_visit_order(w.ring_P, w.ring_C, w.ring_rank)
    else:
        order, members = list(range(w.n_chunks)), None
    gen_s = time.time() - t0

    # ---- resident outputs and workspaces (allocated once, outside the timed region) -----------------
    dev = q.device
    o_acc = torch.empty((w.B, w.Sq, w.Hq, w.D), dtype=torch.float32, device=dev)
    lse = torch.empty((w.B, w.Hq, w.Sq), dtype=torch.float32, device=dev)
    o_low = torch.empty((w.B, w.Sq, w.Hq, w.D), dtype=q.dtype, device=dev)
    ws_f = torch.empty(st.st_ring_workspace_bytes(q, ks, vs, w.q_where, koffs, w.causal, w.scale, mode, False) + 256,
                       dtype=torch.uint8, device=dev)
    if w.backward:
        ws_b = torch.empty(st.st_ring_workspace_bytes(q, ks, vs, w.q_where, koffs, w.causal, w.scale, mode, True) + 256,
                           dtype=torch.uint8, device=dev)
        dq = torch.empty_like(o_acc)
        dkv = torch.empty((2, w.n_chunks) + tuple(ks[0].shape), dtype=torch.float32, device=dev)
        dk = [dkv[0, j] for j in range(w.n_chunks)]
        dv = [dkv[1, j] for j in range(w.n_chunks)]
        dq_low = torch.empty_like(o_low)
        dkv_low = torch.empty(dkv.shape, dtype=q.dtype, device=dev)
        dk_low = [dkv_low[0, j] for j in range(w.n_chunks)]
        dv_low = [dkv_low[1, j] for j in range(w.n_chunks)]

    if team:
        # what the team hands over: the other members' partial states of the same rows (computed here, untimed,
        # by playing those members), and for the backward the team's final O and lse of all gathered rows
        Ct, a_r = w.ring_C, w.ring_rank % w.ring_C
        n_own = w.Sq // Ct
        others = []
        for a in range(Ct):
            if a == a_r:
                continue
            ob = st.st_team_visit_order(w.ring_P, w.ring_C, w.ring_rank - a_r + a)
            o_x, l_x, _ = st.st_ring_fwd(q, ks, vs, w.q_where, koffs, w.causal, w.scale, ob, None, mode,
                                         want_lowp=False, workspace=ws_f)
            others.append((o_x, l_x))
        o_own = torch.empty((w.B, n_own, w.Hq, w.D), dtype=torch.float32, device=dev)
        lse_own = torch.empty((w.B, w.Hq, n_own), dtype=torch.float32, device=dev)
        o_own_low = torch.empty((w.B, n_own, w.Hq, w.D), dtype=q.dtype, device=dev)
        st.st_ring_fwd(q, ks, vs, w.q_where, koffs, w.causal, w.scale, order, None, mode, o_acc=o_acc, lse=lse,
                       want_lowp=False, workspace=ws_f)
        states_o = [o_acc] + [x[0] for x in others]
        states_l = [lse] + [x[1] for x in others]
        o_team, lse_team = st.st_attn_combine(states_o, states_l)
        o_team_low = o_team.to(q.dtype)
        del o_team

    def step_team():
        st.st_ring_fwd(q, ks, vs, w.q_where, koffs, w.causal, w.scale, order, None, mode,
                       o_acc=o_acc, lse=lse, want_lowp=False, workspace=ws_f)
        st.st_attn_combine(states_o, states_l, a_r * n_own, n_own, storage, o_out=o_own, lse_out=lse_own,
                           o_out_lowp=o_own_low)
        if w.backward:
            dq.zero_()
            st.st_ring_bwd_last(q, ks, vs, d_o, o_team_low, lse_team, w.q_where, koffs, w.causal, w.scale, order, dq, dk, dv,
                                assign=True, dk_lowp=dk_low, dv_lowp=dv_low, mode=mode, workspace=ws_b)
            st.st_cast_from_f32(dq, storage, dq_low)

    def step_ring():
        st.st_ring_fwd(q, ks, vs, w.q_where, koffs, w.causal, w.scale, order, members, mode,
                       o_acc=o_acc, lse=lse, o_lowp=o_low, workspace=ws_f)
        if w.backward:
            dq.zero_()
            if bf16:
                # this visit is the chunks' only one: dK / dV are assigned and rounded by the kernels that produce them
                st.st_ring_bwd_last(q, ks, vs, d_o, o_low, lse, w.q_where, koffs, w.causal, w.scale, order, dq, dk, dv,
                                    assign=True, dk_lowp=dk_low, dv_lowp=dv_low, mode=mode, workspace=ws_b)
            else:
                dkv.zero_()
                st.st_ring_bwd(q, ks, vs, d_o, o_low, lse, w.q_where, koffs, w.causal, w.scale, order, dq, dk, dv,
                               mode, workspace=ws_b)
                st.st_cast_from_f32(dkv, storage, dkv_low)
            st.st_cast_from_f32(dq, storage, dq_low)

    step = step_team if team else step_ring
    fwd_flop, bwd_flop = si.algorithmic_flop(w, order if team else None)
    use_graph = args.graph == "on" or (args.graph == "auto" and fwd_flop + bwd_flop < 1e11)
    if use_graph:
        # a launch-bound step (a handful of kernels of some 10 us each) is captured once and replayed: the
        # library only enqueues kernels on the given stream, so the captured graph is the whole step
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()                                   # one-time set-up (device facts) happens outside the capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        eager_step, step = step, graph.replay

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # exactly --steps steps between two synchronisations (host clock: ms_per_step), each one also bracketed by HIP
    # events on the launch stream (median and minimum); the accumulators are re-zeroed inside the step (counted)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(args.steps):
        step()
        ev[i + 1].record()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_each = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps))
    ms_median, ms_min = ms_each[len(ms_each) // 2], ms_each[0]

    # ---- per-kernel durations with HIP events on the launch stream (separate, untimed steps) ---------
    prof_steps = max(1, min(args.steps, 5))
    torch.cuda.synchronize()
    st.st_profile_begin()
    for _ in range(prof_steps):
        (eager_step if use_graph else step)()              # the profiling events are not part of a captured graph
    kernels = st.st_profile_end()

    met = order if team else None                          # chunks that earn FLOP (ring shape: all of them)
    total_flop = fwd_flop + bwd_flop
    value = total_flop / (ms_per_step * 1e-3) / 1e12
    pairs = si.visible_pairs(w, met) * w.Hq * w.B
    # algorithmic work of each MFMA kernel per launch: forward = QK^T and PV; the dK/dV kernel owns
    # S, dP, dV, dK (four of the five backward contractions); the dQ kernel owns dQ (its recomputed
    # S and dP earn nothing)
    algo = {"fwd_bf16": 4 * w.D * pairs, "bwd_dkv_bf16": 8 * w.D * pairs, "bwd_dq_bf16": 2 * w.D * pairs,
            "fwd_f32": 4 * w.D * pairs, "bwd_dkv_f32": 8 * w.D * pairs, "bwd_dq_f32": 2 * w.D * pairs}
    per_kernel = {}
    for name, (launches, total_ms) in kernels.items():
        avg = total_ms / max(launches, 1)
        per_kernel[name] = {"launches_per_step": launches / prof_steps, "avg_ms": round(avg, 4)}
        if name in algo and mode == st.ST_RING_FUSED:
            per_kernel[name]["algorithmic_tflops"] = round(algo[name] / (avg * 1e-3) / 1e12, 1)
    dom = max((n for n in kernels if n in algo), key=lambda n: kernels[n][1], default=None)
    # HIP-event time of the forward and of the backward kernels of a step (the sums of the per-kernel times above)
    fwd_names = {"fwd_bf16", "fwd_edge", "fwd_f32", "combine", "merge"}
    ms_fwd = sum(t for n, (_, t) in kernels.items() if n in fwd_names) / prof_steps
    ms_bwd = sum(t for n, (_, t) in kernels.items() if n not in fwd_names) / prof_steps
    facts = st.st_device_facts()
    # nominal peak from the device the run is on: CUs x 4096 bf16 flop per clock and CU x maximum shader clock
    peak_nominal = facts["compute_units"] * 4096 * facts["max_clock_mhz"] * 1e6 / 1e12 if bf16 else None
    ceiling = mfma_ceiling(st, torch, q) if bf16 else None
    if ceiling and w.D in (64, 128) and mode == st.ST_RING_FUSED:
        # executed MFMA work of each hand-scheduled loop (the dQ loop recomputes S and dP: 6 D per pair for the 2 D it
        # is credited with) against what its instruction mix alone reaches on the workload's data
        mixes = ceiling["workload_q_with_side_instructions"]
        for name, mix, executed_per_credited in (("fwd_bf16", "fwd", 1), ("bwd_dkv_bf16", "dkv", 1), ("bwd_dq_bf16", "dq", 3)):
            if name in per_kernel and "algorithmic_tflops" in per_kernel[name]:
                ex = per_kernel[name]["algorithmic_tflops"] * executed_per_credited
                per_kernel[name]["executed_tflops"] = round(ex, 1)
                per_kernel[name]["frac_of_instruction_mix_ceiling"] = round(ex / mixes[mix + ("64" if w.D == 64 else "")], 3)
    roofline = None
    if dom is not None:
        launches, total_ms = kernels[dom]
        step_ms = total_ms / prof_steps                        # all launches of that kernel in one step
        achieved = algo[dom] / (step_ms * 1e-3) / 1e12
        peak = PEAK_BF16_TFLOPS if bf16 else 157.3
        traffic, traffic_source = hbm_traffic(dom, w.name)
        roofline = {"kernel": dom, "bound": "mfma" if bf16 else "alu", "achieved": round(achieved, 1), "peak": peak,
                    "unit": "TFLOP/s", "frac": round(achieved / peak, 4), "traffic": traffic,
                    "traffic_source": traffic_source,
                    "avg_launch_ms": round(total_ms / max(launches, 1), 4)}
        if ceiling:
            roofline["frac_of_measured_mfma_peak"] = round(achieved / ceiling["workload_q"], 4)

    out = {
        "metric": "fwd+bwd attention TFLOP/s on 1 MI355X + % of bf16 MFMA peak",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_median": round(ms_median, 4), "ms_min": round(ms_min, 4),
        "ms_kernels_by_pass": {"fwd": round(ms_fwd, 4), "bwd": round(ms_bwd, 4)},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D, "Sq": w.Sq, "Sk": w.Sk,
                   "n_chunks": w.n_chunks, "causal": w.causal, "q_offset": w.q_offset, "q_seg": w.q_seg, "q_offset2": w.q_offset2, "mode": args.mode,
                   "shape": args.shape,
                   "visit_order": f"P={w.ring_P},C={w.ring_C},rank={w.ring_rank}" if w.ring_P else "natural",
                   "passes": "fwd+bwd" if w.backward else "fwd", "launch": "hip_graph_replay" if use_graph else "eager"},
        "pct_of_bf16_mfma_peak": round(100.0 * value / PEAK_BF16_TFLOPS, 2),
        "device": {"name": facts["name"], "arch": facts["arch"], "cus": facts["compute_units"], "xcds": facts["xcds"],
                   "max_clock_mhz": facts["max_clock_mhz"], "memory_clock_mhz": facts["memory_clock_mhz"],
                   "memory_bus_bits": facts["memory_bus_bits"], "hbm_gib": round(facts["hbm_bytes"] / 2**30, 1),
                   "host_threads": os.cpu_count()},
        "peak_bf16_tflops": {"divided_by": PEAK_BF16_TFLOPS,
                             "from_device_properties": round(peak_nominal, 1) if peak_nominal else None},
        "measured_mfma_peak_tflops": ceiling,
        "pct_of_measured_mfma_peak": round(100.0 * value / ceiling["workload_q"], 2) if ceiling else None,
        "algorithmic_tflop": {"fwd": round(fwd_flop / 1e12, 4), "bwd": round(bwd_flop / 1e12, 4)},
        "roofline": roofline,
        "kernels": per_kernel,
        "merge_pass": combine_pass(st, torch, states_o, states_l, n_own, w) if team else merge_pass(st, torch, w),
        "input_generation_s": round(gen_s, 1),
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, inp, met)
    print(json.dumps(out))
    return 0


def cpu_baseline(w, inp, met=None) -> dict:
    """The fp64 oracle, as it stands, timed on the host cores on a bounded sample of the same
    workload: forward + backward of a few seeded query rows of the first KV group against all keys
    (team shape: against the keys of the buffers this GPU meets)."""
    import synth_inputs as si
    from oracle import attention as oa

    G = w.Hq // w.Hkv
    heads = list(range(min(G, w.Hq)))                      # the query heads of KV head 0
    met = list(range(w.n_chunks)) if met is None else list(met)
    # about 1e9 (query, key) pairs: some 10 - 15 s of fp64 numpy on the machine's host cores
    rows_per_head = int(max(1, min(w.Sq, 1.1e9 // (len(heads) * w.Sk * len(met)))))
    k_pos = [np.arange(w.Sk, dtype=np.int64) + w.k_offset(j) for j in met]

    def kv_head0(bits_list, f32_list):
        if w.dtype == "bf16":
            return [si.bf16_bits_to_f32(bits_list[j][:, :, 0:1, :]) for j in met]
        return [f32_list[j][:, :, 0:1, :] for j in met]

    k0, v0 = kv_head0(inp.k_bits, inp.k), kv_head0(inp.v_bits, inp.v)
    pairs = 0
    t0 = time.perf_counter()
    for h in heads:
        rows = si.sampled_rows(w, h, rows_per_head)
        q_pos = w.q_positions()[rows]
        qh = inp.q[:, rows, h:h + 1, :]
        oa.attention_forward(qh, k0, v0, q_pos, k_pos, w.causal, w.scale)
        if w.backward:
            oa.attention_backward(qh, k0, v0, inp.d_o[:, rows, h:h + 1, :], q_pos, k_pos, w.causal, w.scale)
        if w.causal:
            pairs += int(sum(np.clip(q_pos - w.k_offset(j) + 1, 0, w.Sk).sum() for j in met))
        else:
            pairs += len(rows) * w.Sk * len(met)
    secs = time.perf_counter() - t0
    flop = (4 + (10 if w.backward else 0)) * w.D * pairs * w.B
    fraction = pairs / max(si.visible_pairs(w, met) * w.Hq, 1)          # of the workload's visible (query, key, head) triples
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": round(flop / secs / 1e12, 6), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"{rows_per_head} seeded query rows of each of {len(heads)} heads (KV head 0) against the "
                      f"{w.Sk * len(met)} keys it meets, fwd{'+bwd' if w.backward else ''}, numpy fp64",
            "seconds": round(secs, 2), "fraction_of_workload": float(f"{fraction:.3e}"),
            "extrapolated_full_seconds": round(secs / fraction, 0)}


if __name__ == "__main__":
    sys.exit(main())
