"""Pins for the fp64 attention oracle (CPU only).

Each test fixes the oracle to something other than itself: closed forms,
invariants of softmax attention, brute-force loops on tiny inputs, a library
routine (torch softmax + autograd in fp64) and central finite differences.
"""
import itertools
import math

import numpy as np
import pytest

from oracle import attention as oa


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def _case(seed=0, B=1, Sq=7, Hq=4, Hkv=2, D=8, lens=(5, 3, 6), q0=None, causal=True):
    N = sum(lens)
    q0 = N - Sq if q0 is None else q0
    q = _rand(seed, B, Sq, Hq, D)
    ks = [_rand(seed + 10 + j, B, L, Hkv, D) for j, L in enumerate(lens)]
    vs = [_rand(seed + 20 + j, B, L, Hkv, D) for j, L in enumerate(lens)]
    d_o = _rand(seed + 30, B, Sq, Hq, D)
    starts = np.concatenate([[0], np.cumsum(lens)])
    kpos = [np.arange(starts[j], starts[j + 1]) for j in range(len(lens))]
    qpos = np.arange(Sq) + q0
    return q, ks, vs, d_o, qpos, kpos, causal, 1.0 / math.sqrt(D)


# ---------------------------------------------------------------- forward pins

def test_softmax_rows_sum_to_one():
    q, ks, vs, _, qpos, kpos, causal, scale = _case(q0=-2)      # rows at positions -2,-1 see nothing
    vs = [np.ones_like(v) for v in vs]
    o, lse = oa.attention_forward(q, ks, vs, qpos, kpos, True, scale)
    assert np.all(o[:, :2] == 0.0) and np.all(np.isneginf(lse[:, :, :2]))
    np.testing.assert_allclose(o[:, 2:], 1.0, rtol=0, atol=1e-14)


@pytest.mark.parametrize("causal", [True, False])
def test_zero_query_gives_log_count_and_mean(causal):
    q, ks, vs, _, qpos, kpos, _, scale = _case(q0=3, lens=(4, 4, 4), Sq=6)
    q = np.zeros_like(q)
    o, lse = oa.attention_forward(q, ks, vs, qpos, kpos, causal, scale)
    v_all = np.concatenate(vs, axis=1)
    G = q.shape[2] // v_all.shape[2]
    for i, p in enumerate(qpos):
        cnt = p + 1 if causal else 12
        np.testing.assert_allclose(lse[0, :, i], math.log(cnt), atol=1e-14)
        for h in range(q.shape[2]):
            np.testing.assert_allclose(o[0, i, h], v_all[0, :cnt, h // G].mean(axis=0), atol=1e-14)


def test_first_token_sees_only_itself():
    q, ks, vs, _, _, kpos, _, scale = _case(lens=(4, 5))
    qpos = np.arange(q.shape[1])                                  # shard starts at global 0
    o, lse = oa.attention_forward(q, ks, vs, qpos, kpos, True, scale)
    G = q.shape[2] // ks[0].shape[2]
    for h in range(q.shape[2]):
        np.testing.assert_allclose(o[0, 0, h], vs[0][0, 0, h // G], atol=1e-15)
        np.testing.assert_allclose(lse[0, h, 0], scale * q[0, 0, h] @ ks[0][0, 0, h // G], atol=1e-14)


def test_one_hot_limit_picks_argmax_key():
    D, N = 8, 8
    k = np.eye(N, D)[None, :, None, :]
    v = _rand(1, 1, N, 1, D)
    pick = np.array([3, 0, 7, 5])
    q = 50.0 * np.eye(N, D)[pick][None, :, None, :]
    o, lse = oa.attention_forward(q, [k], [v], np.full(4, 100), [np.arange(N)], True, 1.0)
    np.testing.assert_allclose(o[0, :, 0], v[0, pick, 0], atol=1e-18 + 8 * math.exp(-50.0) * 4)
    np.testing.assert_allclose(lse[0, 0], 50.0, atol=1e-12)


def test_key_shift_invariance():
    q, ks, vs, _, qpos, kpos, causal, scale = _case()
    c = _rand(99, q.shape[-1])
    o0, l0 = oa.attention_forward(q, ks, vs, qpos, kpos, causal, scale)
    o1, l1 = oa.attention_forward(q, [k + c for k in ks], vs, qpos, kpos, causal, scale)
    np.testing.assert_allclose(o1, o0, atol=1e-13)
    shift = scale * np.einsum("bihd,d->bhi", q, c)
    np.testing.assert_allclose(l1, l0 + shift, atol=1e-12)


def _brute_force(q, ks, vs, qpos, kpos, causal, scale):
    """Explicit loops and math.exp over an explicit (query, key) visibility test."""
    B, Sq, Hq, D = q.shape
    Hkv = ks[0].shape[2]
    G = Hq // Hkv
    o = np.zeros((B, Sq, Hq, D))
    lse = np.full((B, Hq, Sq), -np.inf)
    for b, i, h in itertools.product(range(B), range(Sq), range(Hq)):
        terms = []
        for j, k in enumerate(ks):
            for t in range(k.shape[1]):
                if causal and kpos[j][t] > qpos[i]:
                    continue
                s = scale * sum(q[b, i, h, d] * k[b, t, h // G, d] for d in range(D))
                terms.append((s, vs[j][b, t, h // G]))
        if not terms:
            continue
        z = sum(math.exp(s) for s, _ in terms)
        lse[b, h, i] = math.log(z)
        for s, vrow in terms:
            o[b, i, h] += math.exp(s) / z * vrow
    return o, lse


@pytest.mark.parametrize("causal,q0", [(True, None), (True, 2), (False, 0), (True, -3)])
def test_forward_matches_brute_force(causal, q0):
    q, ks, vs, _, qpos, kpos, _, scale = _case(seed=5, Sq=5, Hq=4, Hkv=2, D=4, lens=(3, 4, 2), q0=q0)
    o, lse = oa.attention_forward(q, ks, vs, qpos, kpos, causal, scale)
    ob, lb = _brute_force(q, ks, vs, qpos, kpos, causal, scale)
    np.testing.assert_allclose(o, ob, atol=1e-13)
    np.testing.assert_allclose(lse, lb, atol=1e-13)


def test_common_offset_shift_changes_nothing():
    q, ks, vs, d_o, qpos, kpos, causal, scale = _case(seed=3)
    a = oa.attention_forward(q, ks, vs, qpos, kpos, causal, scale)
    b = oa.attention_forward(q, ks, vs, qpos + 1000, [p + 1000 for p in kpos], causal, scale)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_future_chunk_contributes_nothing():
    q, ks, vs, d_o, qpos, kpos, causal, scale = _case(seed=4, lens=(5, 3, 6), Sq=4, q0=4)
    # chunk 2 starts at global 8 > last query position 7
    a = oa.attention_forward(q, ks[:2], vs[:2], qpos, kpos[:2], True, scale)
    b = oa.attention_forward(q, ks, vs, qpos, kpos, True, scale)
    np.testing.assert_array_equal(a[0], b[0])
    dq, dk, dv = oa.attention_backward(q, ks, vs, d_o, qpos, kpos, True, scale)
    assert not dk[2].any() and not dv[2].any()


def test_chunk_list_order_is_irrelevant():
    q, ks, vs, d_o, qpos, kpos, causal, scale = _case(seed=6)
    perm = [2, 0, 1]
    a = oa.attention_forward(q, ks, vs, qpos, kpos, causal, scale)
    b = oa.attention_forward(q, [ks[i] for i in perm], [vs[i] for i in perm], qpos,
                             [kpos[i] for i in perm], causal, scale)
    np.testing.assert_allclose(a[0], b[0], atol=1e-14)
    np.testing.assert_allclose(a[1], b[1], atol=1e-14)


def test_gqa_equals_mha_with_repeated_heads():
    q, ks, vs, d_o, qpos, kpos, causal, scale = _case(seed=7, Hq=6, Hkv=2)
    G = 3
    kr = [np.repeat(k, G, axis=2) for k in ks]
    vr = [np.repeat(v, G, axis=2) for v in vs]
    o, lse = oa.attention_forward(q, ks, vs, qpos, kpos, causal, scale)
    o2, lse2 = oa.attention_forward(q, kr, vr, qpos, kpos, causal, scale)
    np.testing.assert_allclose(o, o2, atol=1e-14)
    dq, dk, dv = oa.attention_backward(q, ks, vs, d_o, qpos, kpos, causal, scale)
    dq2, dk2, dv2 = oa.attention_backward(q, kr, vr, d_o, qpos, kpos, causal, scale)
    np.testing.assert_allclose(dq, dq2, atol=1e-13)
    for j in range(len(ks)):
        B, L, _, D = dk2[j].shape
        np.testing.assert_allclose(dk[j], dk2[j].reshape(B, L, 2, G, D).sum(axis=3), atol=1e-13)
        np.testing.assert_allclose(dv[j], dv2[j].reshape(B, L, 2, G, D).sum(axis=3), atol=1e-13)


# --------------------------------------------------------------- library routine

def _torch_reference(q, ks, vs, d_o, qpos, kpos, causal, scale):
    import torch
    tq = torch.tensor(q, dtype=torch.float64, requires_grad=True)
    tk = [torch.tensor(k, dtype=torch.float64, requires_grad=True) for k in ks]
    tv = [torch.tensor(v, dtype=torch.float64, requires_grad=True) for v in vs]
    G = q.shape[2] // ks[0].shape[2]
    k_all = torch.cat(tk, dim=1).repeat_interleave(G, dim=2)
    v_all = torch.cat(tv, dim=1).repeat_interleave(G, dim=2)
    s = torch.einsum("bihd,bthd->bhit", tq, k_all) * scale
    if causal:
        kp = torch.tensor(np.concatenate(kpos))
        qp = torch.tensor(qpos)
        s = s.masked_fill(kp[None, :] > qp[:, None], float("-inf"))
    lse = torch.logsumexp(s, dim=-1)
    o = torch.einsum("bhit,bthd->bihd", torch.softmax(s, dim=-1), v_all)
    (o * torch.tensor(d_o)).sum().backward()
    return (o.detach().numpy(), lse.detach().numpy(), tq.grad.numpy(),
            [k.grad.numpy() for k in tk], [v.grad.numpy() for v in tv])


@pytest.mark.parametrize("causal", [True, False])
def test_against_torch_softmax_and_autograd(causal):
    q, ks, vs, d_o, qpos, kpos, _, scale = _case(seed=11, B=2, Sq=9, Hq=4, Hkv=2, D=16, lens=(7, 4, 8))
    o, lse = oa.attention_forward(q, ks, vs, qpos, kpos, causal, scale)
    dq, dk, dv = oa.attention_backward(q, ks, vs, d_o, qpos, kpos, causal, scale)
    to, tlse, tdq, tdk, tdv = _torch_reference(q, ks, vs, d_o, qpos, kpos, causal, scale)
    np.testing.assert_allclose(o, to, atol=1e-13)
    np.testing.assert_allclose(lse, tlse, atol=1e-13)
    np.testing.assert_allclose(dq, tdq, atol=1e-12)
    for j in range(len(ks)):
        np.testing.assert_allclose(dk[j], tdk[j], atol=1e-12)
        np.testing.assert_allclose(dv[j], tdv[j], atol=1e-12)


# ------------------------------------------------------------------- gradients

def test_gradients_match_central_finite_differences():
    q, ks, vs, d_o, qpos, kpos, causal, scale = _case(seed=21, Sq=4, Hq=4, Hkv=2, D=4, lens=(3, 3), q0=1)
    dq, dk, dv = oa.attention_backward(q, ks, vs, d_o, qpos, kpos, causal, scale)

    def loss():
        return (oa.attention_forward(q, ks, vs, qpos, kpos, causal, scale)[0] * d_o).sum()

    h = 1e-5
    rng = np.random.default_rng(0)
    for arr, grad in [(q, dq)] + list(zip(ks, dk)) + list(zip(vs, dv)):
        for _ in range(12):
            idx = tuple(rng.integers(0, n) for n in arr.shape)
            old = arr[idx]
            arr[idx] = old + h
            lp = loss()
            arr[idx] = old - h
            lm = loss()
            arr[idx] = old
            assert abs((lp - lm) / (2 * h) - grad[idx]) <= 1e-8 * max(1.0, abs(grad[idx]))


def test_gradient_invariants():
    q, ks, vs, d_o, qpos, kpos, causal, scale = _case(seed=22, q0=-1)   # row 0 sees nothing
    dq, dk, dv = oa.attention_backward(q, ks, vs, d_o, qpos, kpos, causal, scale)
    G = q.shape[2] // ks[0].shape[2]
    # softmax is invariant to a common shift of all keys: sum_t dK_t = 0
    np.testing.assert_allclose(sum(x.sum(axis=1) for x in dk), 0.0, atol=1e-13)
    # rows of P sum to one over the visible set: sum_t dV_t = sum over non-empty rows of dO
    want = d_o[:, 1:].sum(axis=1).reshape(1, ks[0].shape[2], G, -1).sum(axis=2)
    np.testing.assert_allclose(sum(x.sum(axis=1) for x in dv), want, atol=1e-13)
    assert not dq[:, 0].any()
    # identical keys: scores do not depend on q, so dQ = 0
    ks_same = [np.broadcast_to(ks[0][:, :1], k.shape).copy() for k in ks]
    dq2, _, _ = oa.attention_backward(q, ks_same, vs, d_o, qpos, kpos, causal, scale)
    np.testing.assert_allclose(dq2, 0.0, atol=1e-14)


# ----------------------------------------------------------- schedule's own steps

def test_merge_is_commutative_associative_with_identity():
    q, ks, vs, _, qpos, kpos, causal, scale = _case(seed=31, q0=2)
    parts = [oa.block_forward(q, k, v, qpos, p, causal, scale) for k, v, p in zip(ks, vs, kpos)]
    ab = oa.merge(*parts[0], *parts[1])
    ba = oa.merge(*parts[1], *parts[0])
    np.testing.assert_allclose(ab[0], ba[0], atol=1e-15)
    l = oa.merge(*ab, *parts[2])
    r = oa.merge(*parts[0], *oa.merge(*parts[1], *parts[2]))
    np.testing.assert_allclose(l[0], r[0], atol=1e-14)
    np.testing.assert_allclose(l[1], r[1], atol=1e-14)
    e = oa.empty_state(*q.shape)
    m = oa.merge(*e, *parts[2])           # chunk 2 is invisible to the first rows: -inf meets -inf
    assert np.array_equal(m[0], parts[2][0]) and np.array_equal(m[1], parts[2][1])
    assert not np.isnan(m[0]).any() and not np.isnan(m[1]).any()


def test_merge_of_two_single_keys_closed_form():
    # two one-key states: lse are the scores, O the value rows -> 2-way softmax
    o_a, o_b = np.full((1, 1, 1, 2), 3.0), np.full((1, 1, 1, 2), -1.0)
    l_a, l_b = np.full((1, 1, 1), 0.5), np.full((1, 1, 1), -0.25)
    o, lse = oa.merge(o_a, l_a, o_b, l_b)
    wa = 1.0 / (1.0 + math.exp(-0.75))
    np.testing.assert_allclose(o, wa * 3.0 + (1 - wa) * -1.0, atol=1e-15)
    np.testing.assert_allclose(lse, math.log(math.exp(0.5) + math.exp(-0.25)), atol=1e-15)


def test_combine_of_single_keys_closed_form():
    # three one-key states: lse are the scores, O the value rows -> a 3-way softmax written out
    scores, values = [0.5, -0.25, 1.5], [3.0, -1.0, 0.25]
    o_parts = [np.full((1, 1, 1, 2), v) for v in values]
    l_parts = [np.full((1, 1, 1), s) for s in scores]
    o, lse = oa.combine(o_parts, l_parts)
    z = sum(math.exp(s) for s in scores)
    np.testing.assert_allclose(o, sum(math.exp(s) / z * v for s, v in zip(scores, values)), atol=1e-15)
    np.testing.assert_allclose(lse, math.log(z), atol=1e-15)


@pytest.mark.parametrize("causal", [True, False])
def test_combine_of_key_subsets_equals_monolithic(causal):
    """Partial states over disjoint key subsets (what the team members hold), combined in one pass, are the
    attention over all keys; only the asked rows come back; the order of the states is irrelevant."""
    q, ks, vs, _, qpos, kpos, _, scale = _case(seed=34, lens=(5, 3, 6, 2, 4), Sq=9, q0=8)
    o, lse = oa.attention_forward(q, ks, vs, qpos, kpos, causal, scale)
    groups = [[0, 3], [1], [4, 2]]
    parts = [oa.attention_forward(q, [ks[j] for j in g], [vs[j] for j in g], qpos, [kpos[j] for j in g], causal, scale)
             for g in groups]
    oc, lc = oa.combine([p[0] for p in parts], [p[1] for p in parts])
    np.testing.assert_allclose(oc, o, atol=1e-13)
    np.testing.assert_allclose(lc, lse, atol=1e-13)
    for perm in itertools.permutations(range(3)):
        op, lp = oa.combine([parts[x][0] for x in perm], [parts[x][1] for x in perm], row0=2, n_rows=5)
        np.testing.assert_allclose(op, o[:, 2:7], atol=1e-13)
        np.testing.assert_allclose(lp, lse[:, :, 2:7], atol=1e-13)


def test_combine_special_cases():
    q, ks, vs, _, qpos, kpos, causal, scale = _case(seed=35, q0=2)
    parts = [oa.block_forward(q, k, v, qpos, p, causal, scale) for k, v, p in zip(ks, vs, kpos)]
    # one state: identity;  two states: the pairwise merge;  empty states change nothing
    o1, l1 = oa.combine([parts[0][0]], [parts[0][1]])
    assert np.array_equal(o1, parts[0][0]) and np.array_equal(l1, parts[0][1])
    o2, l2 = oa.combine([parts[0][0], parts[1][0]], [parts[0][1], parts[1][1]])
    om, lm = oa.merge(*parts[0], *parts[1])
    np.testing.assert_allclose(o2, om, atol=1e-15)
    np.testing.assert_allclose(l2, lm, atol=1e-15)
    e = oa.empty_state(*q.shape)
    o3, l3 = oa.combine([e[0], parts[0][0], e[0], parts[1][0]], [e[1], parts[0][1], e[1], parts[1][1]])
    np.testing.assert_allclose(o3, om, atol=1e-15)
    np.testing.assert_allclose(l3, lm, atol=1e-15)
    o4, l4 = oa.combine([e[0], e[0]], [e[1], e[1]])
    assert np.array_equal(o4, e[0]) and np.array_equal(l4, e[1]) and not np.isnan(o4).any()


@pytest.mark.parametrize("causal", [True, False])
def test_blockwise_merge_equals_monolithic_for_any_order(causal):
    q, ks, vs, d_o, qpos, kpos, _, scale = _case(seed=32, lens=(5, 3, 6, 2), Sq=8, q0=6)
    o, lse = oa.attention_forward(q, ks, vs, qpos, kpos, causal, scale)
    for order in ([0, 1, 2, 3], [3, 2, 1, 0], [2, 0, 3, 1]):
        for members in (None, [0, 0, 1, 1], [1, 0, 1, 0]):
            ob, lb = oa.ring_forward(q, ks, vs, qpos, kpos, causal, scale, order, members)
            np.testing.assert_allclose(ob, o, atol=1e-13)
            np.testing.assert_allclose(lb, lse, atol=1e-13)


def test_blockwise_backward_equals_monolithic():
    q, ks, vs, d_o, qpos, kpos, causal, scale = _case(seed=33, lens=(5, 3, 6, 2), Sq=8, q0=6)
    o, lse = oa.attention_forward(q, ks, vs, qpos, kpos, causal, scale)
    dq, dk, dv = oa.attention_backward(q, ks, vs, d_o, qpos, kpos, causal, scale)
    dq2, dk2, dv2 = oa.ring_backward(q, ks, vs, d_o, o, lse, qpos, kpos, causal, scale, [2, 0, 3, 1])
    np.testing.assert_allclose(dq2, dq, atol=1e-13)
    for j in range(4):
        np.testing.assert_allclose(dk2[j], dk[j], atol=1e-13)
        np.testing.assert_allclose(dv2[j], dv[j], atol=1e-13)


def test_delta_is_rowsum():
    d_o, o = _rand(1, 2, 3, 4, 5), _rand(2, 2, 3, 4, 5)
    dl = oa.delta(d_o, o)
    assert dl.shape == (2, 4, 3)
    assert dl[1, 2, 0] == pytest.approx(float(np.dot(d_o[1, 0, 2], o[1, 0, 2])), abs=1e-15)


# ------------------------------------------------ planted mistakes must be caught

def test_pins_catch_a_transposed_or_dropped_term(monkeypatch):
    """Sanity of the pins themselves: plant typical mistakes in the oracle (on the
    CPU) and check that the finite-difference / torch pins would fail."""
    q, ks, vs, d_o, qpos, kpos, causal, scale = _case(seed=41)
    ref = _torch_reference(q, ks, vs, d_o, qpos, kpos, causal, scale)

    real_probs = oa._probs
    monkeypatch.setattr(oa, "_probs", lambda s, lse: real_probs(s, lse) * 1.0001)
    o_bad, _ = oa.attention_forward(q, ks, vs, qpos, kpos, causal, scale)
    assert np.abs(o_bad - ref[0]).max() > 1e-6
    monkeypatch.setattr(oa, "_probs", real_probs)

    real_vis = oa._visible
    monkeypatch.setattr(oa, "_visible", lambda a, b, c: real_vis(a - 1, b, c))      # exclusive diagonal
    o_bad, _ = oa.attention_forward(q, ks, vs, qpos, kpos, causal, scale)
    assert np.abs(o_bad - ref[0]).max() > 1e-3
