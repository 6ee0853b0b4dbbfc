"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its
host logic (visit order, validation that fails before any launch) behaves."""
import ctypes as C
import os
import re

import pytest

import paper_2407_00611_amd as st
from paper_2407_00611_amd import api
from oracle import visit_order as ov

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "startrail.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(st_[a-z0-9_]+)\s*\(", header))
    assert declared == set(api.EXPORTS)
    lib = C.CDLL(st.library_path())
    for name in declared:
        assert hasattr(lib, name), name


def test_version_and_strings():
    assert st.st_version() >= 100
    assert st.st_status_str(0) == "ok"
    assert "alignment" in st.st_status_str(3) or "misaligned" in st.st_status_str(3)


@pytest.mark.parametrize("P,C", [(1, 1), (4, 1), (4, 2), (8, 2), (16, 1), (16, 2), (16, 4), (32, 2), (32, 4),
                                 (64, 1), (64, 2), (64, 4), (64, 8), (36, 3), (54, 3)])
def test_visit_order_matches_cluster_simulation(P, C):
    for rank in range(P):
        assert st.st_visit_order(P, C, rank) == ov.visit_order(P, C, rank)


@pytest.mark.parametrize("P,C", [(1, 1), (4, 1), (4, 2), (8, 2), (16, 2), (16, 4), (32, 2), (32, 4), (64, 2), (64, 4),
                                 (64, 8), (36, 3), (54, 3)])
def test_team_visit_order_matches_cluster_simulation(P, C):
    for rank in range(P):
        assert st.st_team_visit_order(P, C, rank) == ov.team_visit_order(P, C, rank)


def test_team_visit_order_rejects_bad_layouts():
    for P, C, r in [(8, 3, 0), (8, 4, 0), (0, 1, 0), (8, 0, 0), (12, 4, 0), (8, 2, 8), (8, 2, -1)]:
        with pytest.raises(st.StarTrailError) as e:
            st.st_team_visit_order(P, C, r)
        assert e.value.status == 1


def test_two_run_placements_are_validated():
    """Second run of query rows: inside the shard, and not before the end of the first run."""
    for bad in [dict(q_seg=8, q_offset2=100), dict(q_seg=-1, q_offset2=100), dict(q_seg=9, q_offset2=100),
                dict(q_seg=4, q_offset2=3), dict(q_offset=10, q_seg=4, q_offset2=13)]:
        assert _call_fwd(_desc(**bad)) == 1, bad


def test_combine_validation_fails_before_any_launch():
    lib = api._lib
    def call(n=2, B=1, Sq_in=8, Hq=2, D=64, row0=0, Sq_out=8, o=(0x1000, 0x2000), l=(0x3000, 0x4000), out=0x5000,
             lout=0x6000, dtype=0, low=None):
        op = (C.c_void_p * len(o))(*o)
        lp = (C.c_void_p * len(l))(*l)
        return lib.st_attn_combine(op, lp, n, B, Sq_in, Hq, D, row0, Sq_out, C.c_void_p(out), C.c_void_p(lout), dtype,
                                   C.c_void_p(low) if low else None, None)
    assert call(n=0) == 1 and call(n=65) == 1
    assert call(row0=1) == 1 and call(row0=-1) == 1 and call(Sq_out=9) == 1
    assert call(D=260) == 2 and call(D=12) == 2
    assert call(o=(0x1000, 0x2004)) == 3 and call(o=(0x1000, 0)) == 1
    assert call(out=0x1000) == 1 and call(dtype=7) == 1 and call(low=0x7008, dtype=1) == 3
    assert call(Sq_out=0, row0=8) == 0 and call(B=0) == 0          # nothing to do: no launch


def test_visit_order_rejects_bad_layouts():
    for P, C, r in [(8, 3, 0), (8, 4, 0), (0, 1, 0), (8, 0, 0), (12, 4, 0), (8, 2, 8), (8, 2, -1)]:
        with pytest.raises(st.StarTrailError) as e:
            st.st_visit_order(P, C, r)
        assert e.value.status == 1


def _desc(**kw):
    base = dict(dtype=0, B=1, Hq=2, Hkv=1, D=64, Sq=8, Sk=8, q_offset=0, k_offset=0, causal=1, scale=0.125, q_seg=0,
                q_offset2=0)
    base.update(kw)
    return api.st_block_desc(*[base[k] for k, _ in api.st_block_desc._fields_])


def _call_fwd(desc, q=0x1000, k=0x2000, v=0x3000, o=0x4000, lse=0x5000, strides=(1024, 128, 64)):
    lib = api._lib
    tq, tk, tv = (api.st_tensor(p, *strides) for p in (q, k, v))
    return lib.st_attn_block_fwd(C.byref(desc), C.byref(tq), C.byref(tk), C.byref(tv), C.c_void_p(o),
                                 C.c_void_p(lse), None)


def test_validation_fails_before_any_launch():
    """Fake device pointers: every call below must be rejected on the host."""
    assert _call_fwd(_desc(Hq=3, Hkv=2)) == 1                 # Hq % Hkv
    assert _call_fwd(_desc(dtype=7)) == 1
    assert _call_fwd(_desc(Sq=-1)) == 1
    assert _call_fwd(_desc(D=512)) == 2                        # no kernel
    assert _call_fwd(_desc(dtype=1, D=96)) == 2
    assert _call_fwd(_desc(), q=0x1004) == 3                   # misaligned base
    assert _call_fwd(_desc(), strides=(1024, 130, 64)) == 3    # misaligned row stride
    assert _call_fwd(_desc(), k=0) == 1                        # null
    assert "null" in st.st_last_error()
    assert api._lib.st_attn_block_fwd(None, None, None, None, None, None, None) == 1
    assert api._lib.st_attn_merge(C.c_void_p(0x1000), C.c_void_p(0x2000), C.c_void_p(0x1000), C.c_void_p(0x3000),
                                  1, 8, 2, 64, 0, None, None) == 1      # o_part aliases o_acc
    assert api._lib.st_attn_merge(C.c_void_p(0x1000), C.c_void_p(0x2000), C.c_void_p(0x3000), C.c_void_p(0x4000),
                                  1, 8, 2, 60, 0, None, None) == 2
    assert api._lib.st_cast_from_f32(C.c_void_p(0x1000), C.c_void_p(0x2002), 16, 1, None) == 3


def test_empty_problems_are_ok_without_a_gpu():
    assert _call_fwd(_desc(Sq=0), q=0, o=0, lse=0) == 0
    assert _call_fwd(_desc(B=0), q=0, k=0, v=0, o=0, lse=0) == 0


def test_forward_workspace_covers_every_visited_subset():
    """An under-filled fused forward is split over the visited chunks; the workspace the library asks for must be
    enough for any subset of the table the caller may then visit (host logic only: no launch)."""
    import torch

    def need(n_chunks, Sq=300, Hq=2, D=128, Sk=64):
        q = torch.zeros((1, Sq, Hq, D), dtype=torch.bfloat16)
        ks = [torch.zeros((1, Sk, 1, D), dtype=torch.bfloat16) for _ in range(n_chunks)]
        return st.st_ring_workspace_bytes(q, ks, ks, 0, [Sk * j for j in range(n_chunks)], True, 0.1, st.ST_RING_FUSED, False)

    one = need(1)
    assert one > 0 and need(2) == 3 * one                    # two chunks: a state per split and the general workgroups' own
    sizes = [need(n) for n in (1, 2, 5, 16, 50, 64)]
    assert sizes == sorted(sizes)                             # grows with the table ...
    assert need(150) == need(64) == need(256)                 # ... up to one launch's table, and stays there
    assert need(64, Sq=4096, Hq=32) == need(1, Sq=4096, Hq=32)  # enough query tiles to fill the chip: never split


def test_ring_bwd_last_validation_fails_before_any_launch():
    """Fake device pointers: the arguments st_ring_bwd_last adds are checked on the host."""
    lib = api._lib
    n = 2
    k_ptr = (C.c_void_p * n)(0x10000, 0x20000)
    v_ptr = (C.c_void_p * n)(0x30000, 0x40000)
    k_off = (C.c_int64 * n)(0, 8)
    vpp = C.POINTER(C.c_void_p)

    def desc(dtype):
        return api.st_ring_desc(dtype, 1, 2, 1, 64, 8, 8, 16, 1, 0.125, n, C.cast(k_ptr, vpp), C.cast(v_ptr, vpp),
                                512, 64, 64, 512, 64, 64, C.cast(k_off, C.POINTER(C.c_int64)), 0, 0)

    def call(dtype=1, flags=0, lk=None, lv=None, ws=0x900000, ws_bytes=1 << 20):
        d = desc(dtype)
        t = api.st_tensor(0x1000, 1024, 128, 64)
        order = (C.c_int32 * n)(0, 1)
        dk = (C.c_void_p * n)(0x50000, 0x60000)
        dv = (C.c_void_p * n)(0x70000, 0x80000)
        return lib.st_ring_bwd_last(C.byref(d), C.byref(t), C.byref(t), C.byref(t), dtype, C.c_void_p(0x2000), order, n, 1,
                                    C.c_void_p(0x3000), C.cast(dk, vpp), C.cast(dv, vpp), flags,
                                    C.cast(lk, vpp) if lk is not None else None, C.cast(lv, vpp) if lv is not None else None,
                                    C.c_void_p(ws), ws_bytes, None)

    both = (C.c_void_p * n)(0xa0000, 0xb0000)
    half = (C.c_void_p * n)(0xa0000, None)
    odd = (C.c_void_p * n)(0xa0004, 0xb0000)
    assert call(flags=2) == 1 and "kv_flags" in st.st_last_error()
    assert call(lk=both) == 1                                  # one table without the other
    assert call(lk=both, lv=half) == 1                         # one entry without the other
    assert call(lk=odd, lv=both) == 3                          # misaligned copy
    assert call(dtype=0, lk=both, lv=both) == 2                # bf16 copies of an fp32 problem
    assert call(flags=1, lk=both, lv=both, ws=0) == 5          # arguments fine: stops at the missing workspace


def test_mfma_probe_mixes_and_validation():
    """The benchmark probe: its mixes have names, and bad arguments fail before any launch."""
    n = api.st_mfma_probe_mixes()
    names = [api.st_mfma_probe_mix_name(m) for m in range(n + 1)]
    assert names[0] == "none" and len(set(names)) == n + 1 and all(names)
    assert {"fwd", "dq", "dkv", "fwd64", "dq64", "dkv64"} <= set(names)
    assert api.st_mfma_probe_mix_name(n + 1) == "" and api.st_mfma_probe_mix_name(-1) == ""
    flop = C.c_double(-1.0)

    def call(ops=0x10000, nbytes=1 << 20, mix=0, iters=10, sink=0x20000, nsink=1 << 20):
        return api._lib.st_mfma_probe(C.c_void_p(ops), nbytes, mix, iters, C.cast(C.c_void_p(sink), C.POINTER(C.c_float)),
                                      nsink, C.byref(flop), None)

    assert call(ops=0) == 1 and call(sink=0) == 1
    assert call(ops=0x10008) == 3                       # not 16-byte aligned
    assert call(nbytes=4096) == 1 and call(iters=0) == 1 and call(iters=(1 << 24) + 1) == 1
    assert call(mix=-1) == 1 and call(mix=n + 1) == 1
    assert call(nsink=16) == 1                          # the sink holds one float per thread of the launch
    assert flop.value == -1.0
