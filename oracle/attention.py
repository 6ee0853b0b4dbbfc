"""CPU oracle for one GPU's share of ring attention (fp64, numpy).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the HIP
kernels are checked against.  It shares no code with the library under
``paper_2407_00611_amd/`` and nothing in the library may import it.

What it computes.  The ring / concentric-ring schedule delivers KV chunks to a
resident query shard step by step and folds each step into a running
``(O, lse)`` state (Algorithm 1, the ``forward_iteration`` step and the final
``ReduceScatter_combine``); the paper states that this leaves the computation
result unchanged (abstract; Section 3.2).  The result therefore has a plain
definition -- softmax attention of the query shard over *all* delivered keys
(Section 2.1, the scaled dot-product attention equation) -- and the main
oracle below is that definition written out monolithically: no tiling, no
online softmax, no dependence on the visit order.

A second group of functions follows the schedule's own steps in the paper's
order (per-chunk attention, log-sum-exp merge, per-chunk backward from the
final statistics, Section 3.2 "Forward Propagation" / "Backward Propagation").
They exist so the step-level entry points of the library can be compared
one by one, and so that the identity "blockwise + merge == monolithic" is
checked on the CPU before any GPU code runs.

Conventions (where the paper is silent the reading is stated here):
  * q, d_o: [B, Sq, Hq, D]; each KV chunk: [B, Sk_j, Hkv, D]; O like q;
    LSE, delta: [B, Hq, Sq].  Query head h reads KV head h // (Hq // Hkv).
  * q_pos[i] / k_pos[t] are *global* token positions.  Causal: key visible
    iff k_pos <= q_pos (diagonal inclusive).  Non-causal: every key visible.
  * LSE is the natural log of sum(exp(scale * <q, k>)) over visible keys.
  * A row with no visible key has O = 0, LSE = -inf and contributes no gradient.
  * Gradients are those of L = sum(O * d_o) with d_o fixed (LSE has no cotangent).
All arithmetic is fp64; inputs of any float dtype are widened exactly.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

NEG_INF = -np.inf


def _f64(x) -> np.ndarray:
    return np.asarray(x, dtype=np.float64)


def _visible(q_pos: np.ndarray, k_pos: np.ndarray, causal: bool) -> np.ndarray:
    """Boolean [Sq, Nk]: may query i look at key t?  (global positions)"""
    if not causal:
        return np.ones((len(q_pos), len(k_pos)), dtype=bool)
    return np.asarray(k_pos)[None, :] <= np.asarray(q_pos)[:, None]


def _scores(qh: np.ndarray, kh: np.ndarray, vis: np.ndarray, scale: float) -> np.ndarray:
    """scale * q k^T with -inf where masked.  qh [Sq,D], kh [Nk,D]."""
    s = scale * (qh @ kh.T)
    s[~vis] = NEG_INF
    return s


def _lse_rows(s: np.ndarray) -> np.ndarray:
    """Row-wise log-sum-exp; -inf for rows that are entirely -inf."""
    m = s.max(axis=1) if s.shape[1] else np.full(s.shape[0], NEG_INF)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    with np.errstate(divide="ignore"):
        lse = m_safe + np.log(np.exp(s - m_safe[:, None]).sum(axis=1))
    return np.where(np.isfinite(m), lse, NEG_INF)


def _probs(s: np.ndarray, lse: np.ndarray) -> np.ndarray:
    """P = exp(s - lse) row-wise; rows with lse = -inf give all zeros."""
    lse_safe = np.where(np.isfinite(lse), lse, 0.0)
    p = np.exp(s - lse_safe[:, None])
    p[~np.isfinite(lse), :] = 0.0
    return p


# ==========================================================================
# Monolithic definition (Section 2.1 attention equation; abstract: the
# schedule does not change the result)
# ==========================================================================

def attention_forward(q, k_chunks: Sequence, v_chunks: Sequence, q_pos, k_pos_chunks: Sequence,
                      causal: bool, scale: float) -> Tuple[np.ndarray, np.ndarray]:
    """Softmax attention of the query shard over the union of all chunks.

    Returns O [B,Sq,Hq,D] and LSE [B,Hq,Sq] (fp64).  The order of the chunks
    in the lists is irrelevant by construction (they are concatenated)."""
    B, Sq, Hq, D = q.shape
    Hkv = k_chunks[0].shape[2]
    G = Hq // Hkv
    q_pos = np.asarray(q_pos, dtype=np.int64)
    k_pos = np.concatenate([np.asarray(p, dtype=np.int64) for p in k_pos_chunks])
    vis = _visible(q_pos, k_pos, causal)
    O = np.zeros((B, Sq, Hq, D))
    LSE = np.full((B, Hq, Sq), NEG_INF)
    for b in range(B):
        for g in range(Hkv):
            kh = np.concatenate([_f64(k[b, :, g, :]) for k in k_chunks], axis=0)
            vh = np.concatenate([_f64(v[b, :, g, :]) for v in v_chunks], axis=0)
            for h in range(g * G, (g + 1) * G):
                s = _scores(_f64(q[b, :, h, :]), kh, vis, scale)
                lse = _lse_rows(s)
                p = _probs(s, lse)
                O[b, :, h, :] = p @ vh
                LSE[b, h, :] = lse
    return O, LSE


def attention_backward(q, k_chunks: Sequence, v_chunks: Sequence, d_o, q_pos,
                       k_pos_chunks: Sequence, causal: bool, scale: float):
    """Gradients of L = sum(O * d_o) w.r.t. q and every chunk's k and v.

    Differentiating O_i = sum_t P_it v_t, P = softmax(s), s = scale q k^T:
      dV_t = sum_i P_it dO_i
      dP_it = <dO_i, v_t>;  dS_it = P_it (dP_it - Delta_i),  Delta_i = <dO_i, O_i>
      dQ_i = scale sum_t dS_it k_t;  dK_t = scale sum_i dS_it q_i
    with dK, dV summed over the query heads that share a KV head.
    Returns dQ [B,Sq,Hq,D], [dK_j], [dV_j] (fp64, this shard's contribution)."""
    B, Sq, Hq, D = q.shape
    Hkv = k_chunks[0].shape[2]
    G = Hq // Hkv
    lens = [k.shape[1] for k in k_chunks]
    starts = np.concatenate([[0], np.cumsum(lens)])
    q_pos = np.asarray(q_pos, dtype=np.int64)
    k_pos = np.concatenate([np.asarray(p, dtype=np.int64) for p in k_pos_chunks])
    vis = _visible(q_pos, k_pos, causal)
    dQ = np.zeros((B, Sq, Hq, D))
    dK_all = np.zeros((B, int(starts[-1]), Hkv, D))
    dV_all = np.zeros_like(dK_all)
    for b in range(B):
        for g in range(Hkv):
            kh = np.concatenate([_f64(k[b, :, g, :]) for k in k_chunks], axis=0)
            vh = np.concatenate([_f64(v[b, :, g, :]) for v in v_chunks], axis=0)
            for h in range(g * G, (g + 1) * G):
                qh = _f64(q[b, :, h, :])
                doh = _f64(d_o[b, :, h, :])
                s = _scores(qh, kh, vis, scale)
                p = _probs(s, _lse_rows(s))
                oh = p @ vh
                delta = (doh * oh).sum(axis=1)
                d_p = doh @ vh.T
                d_s = p * (d_p - delta[:, None])
                dQ[b, :, h, :] = scale * (d_s @ kh)
                dK_all[b, :, g, :] += scale * (d_s.T @ qh)
                dV_all[b, :, g, :] += p.T @ doh
    dK = [dK_all[:, starts[j]:starts[j + 1]] for j in range(len(lens))]
    dV = [dV_all[:, starts[j]:starts[j + 1]] for j in range(len(lens))]
    return dQ, dK, dV


# ==========================================================================
# The schedule's own steps (Algorithm 1; Section 3.2 forward / backward text)
# ==========================================================================

def block_forward(q, k, v, q_pos, k_pos, causal: bool, scale: float):
    """One ``forward_iteration`` before its fold: attention of the query shard
    against ONE chunk.  Returns the partial (O_part, lse_part)."""
    return attention_forward(q, [k], [v], q_pos, [k_pos], causal, scale)


def merge(o_a, lse_a, o_b, lse_b):
    """Fold two partial states for the same query rows (the online-softmax
    update of ``forward_iteration`` and the arithmetic of
    ``ReduceScatter_combine``):
        lse' = log(exp(lse_a) + exp(lse_b))
        O'   = exp(lse_a - lse') O_a + exp(lse_b - lse') O_b
    o_*: [B,Sq,Hq,D]; lse_*: [B,Hq,Sq].  A state with lse = -inf is empty and
    acts as the identity."""
    o_a, o_b, lse_a, lse_b = _f64(o_a), _f64(o_b), _f64(lse_a), _f64(lse_b)
    m = np.maximum(lse_a, lse_b)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    with np.errstate(divide="ignore"):
        lse = m_safe + np.log(np.exp(lse_a - m_safe) + np.exp(lse_b - m_safe))
    lse = np.where(np.isfinite(m), lse, NEG_INF)
    lse_safe = np.where(np.isfinite(lse), lse, 0.0)
    w_a = np.where(np.isfinite(lse_a), np.exp(lse_a - lse_safe), 0.0)   # [B,Hq,Sq]
    w_b = np.where(np.isfinite(lse_b), np.exp(lse_b - lse_safe), 0.0)
    o = w_a.transpose(0, 2, 1)[..., None] * o_a + w_b.transpose(0, 2, 1)[..., None] * o_b
    return o, lse


def combine(o_parts: Sequence, lse_parts: Sequence, row0: int = 0, n_rows: int = None):
    """``ReduceScatter_combine`` of Algorithm 1 written as its definition: n partial
    states of the same query rows, each over a different part of the keys, and
    the run of rows [row0, row0 + n_rows) that is kept:
        lse' = log(sum_x exp(lse_x)),   O' = sum_x exp(lse_x - lse') O_x
    An empty state (lse = -inf) contributes nothing; a row empty in every state
    gives O = 0 and lse = -inf.  o_x: [B,Sq,Hq,D]; lse_x: [B,Hq,Sq]."""
    o_parts = [_f64(o) for o in o_parts]
    lse_parts = [_f64(l) for l in lse_parts]
    Sq = o_parts[0].shape[1]
    n_rows = Sq - row0 if n_rows is None else n_rows
    rows = slice(row0, row0 + n_rows)
    lse_stack = np.stack([l[:, :, rows] for l in lse_parts])              # [n,B,Hq,rows]
    m = lse_stack.max(axis=0)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    with np.errstate(divide="ignore"):
        lse = m_safe + np.log(np.exp(lse_stack - m_safe).sum(axis=0))
    lse = np.where(np.isfinite(m), lse, NEG_INF)
    lse_safe = np.where(np.isfinite(lse), lse, 0.0)
    o = np.zeros_like(o_parts[0][:, rows])
    for o_x, l_x in zip(o_parts, lse_stack):
        w = np.where(np.isfinite(l_x), np.exp(l_x - lse_safe), 0.0)       # [B,Hq,rows]
        o += w.transpose(0, 2, 1)[..., None] * o_x[:, rows]
    return o, lse


def empty_state(B: int, Sq: int, Hq: int, D: int):
    """Initial running state: O = 0 and lse = -inf (the neutral element of merge)."""
    return np.zeros((B, Sq, Hq, D)), np.full((B, Hq, Sq), NEG_INF)


def ring_forward(q, k_chunks, v_chunks, q_pos, k_pos_chunks, causal, scale,
                 order: Sequence[int], member_of: Sequence[int] = None):
    """Walk the chunks in ``order`` as the ring would deliver them.  Each
    simulated team member keeps its own running state (its sub-ring iterations);
    the member states are combined at the end (``ReduceScatter_combine``)."""
    B, Sq, Hq, D = q.shape
    if member_of is None:
        member_of = [0] * len(order)
    states = {}
    for j, mem in zip(order, member_of):
        o_p, l_p = block_forward(q, k_chunks[j], v_chunks[j], q_pos, k_pos_chunks[j], causal, scale)
        o_s, l_s = states.get(mem, empty_state(B, Sq, Hq, D))
        states[mem] = merge(o_s, l_s, o_p, l_p)
    o, lse = empty_state(B, Sq, Hq, D)
    for mem in sorted(states):
        o, lse = merge(o, lse, *states[mem])
    return o, lse


def delta(d_o, o) -> np.ndarray:
    """Delta[b,h,i] = <dO_i, O_i> with the FINAL merged O (saved at the
    attention output, Section "StarTrail Runtime": checkpoint placement)."""
    return (_f64(d_o) * _f64(o)).sum(axis=-1).transpose(0, 2, 1)


def block_backward(q, k, v, d_o, lse_final, delta_final, q_pos, k_pos, causal: bool, scale: float):
    """One backward iteration: the query shard (with its final lse and Delta)
    meets ONE resident chunk.  Returns this pair's dQ contribution (to be
    added to the circulating dQ) and the chunk's dK, dV contributions."""
    B, Sq, Hq, D = q.shape
    Hkv = k.shape[2]
    G = Hq // Hkv
    vis = _visible(np.asarray(q_pos, dtype=np.int64), np.asarray(k_pos, dtype=np.int64), causal)
    dQ = np.zeros((B, Sq, Hq, D))
    dK = np.zeros((B, k.shape[1], Hkv, D))
    dV = np.zeros_like(dK)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            qh, kh, vh, doh = _f64(q[b, :, h]), _f64(k[b, :, g]), _f64(v[b, :, g]), _f64(d_o[b, :, h])
            p = _probs(_scores(qh, kh, vis, scale), _f64(lse_final[b, h]))
            d_s = p * (doh @ vh.T - _f64(delta_final[b, h])[:, None])
            dQ[b, :, h] = scale * (d_s @ kh)
            dK[b, :, g] += scale * (d_s.T @ qh)
            dV[b, :, g] += p.T @ doh
    return dQ, dK, dV


def ring_backward(q, k_chunks, v_chunks, d_o, o_final, lse_final, q_pos, k_pos_chunks, causal,
                  scale, order: Sequence[int]):
    """Backward walk: Delta once, then one ``block_backward`` per visited chunk,
    dQ accumulated across chunks, dK/dV staying with their chunk."""
    dl = delta(d_o, o_final)
    dQ = np.zeros(q.shape)
    dK: List = [None] * len(k_chunks)
    dV: List = [None] * len(k_chunks)
    for j in order:
        dq_j, dK[j], dV[j] = block_backward(q, k_chunks[j], v_chunks[j], d_o, lse_final, dl,
                                            q_pos, k_pos_chunks[j], causal, scale)
        dQ += dq_j
    for j in range(len(k_chunks)):
        if dK[j] is None:
            dK[j] = np.zeros(np.asarray(k_chunks[j]).shape)
            dV[j] = np.zeros(np.asarray(v_chunks[j]).shape)
    return dQ, dK, dV
