"""ctypes bindings with the same names as the C ABI in ``include/startrail.h``.

Argument marshalling only: tensors are torch tensors on the GPU ([B, S, heads, D] with D
contiguous, fp32 or bf16), outputs are allocated with torch when not supplied, and every
call is enqueued on torch's current stream.  A non-zero status raises StarTrailError.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import torch

ST_F32, ST_BF16 = 0, 1
ST_RING_STEPWISE, ST_RING_FUSED = 0, 1
ST_KV_ASSIGN = 1
ST_MAX_CHUNKS = 256

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libstartrail.so")


class StarTrailError(RuntimeError):
    def __init__(self, status: int, where: str, text: str):
        super().__init__(f"{where}: status {status} ({text})")
        self.status = status


class st_tensor(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("stride_b", C.c_int64), ("stride_s", C.c_int64), ("stride_h", C.c_int64)]


class st_block_desc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
                ("Sq", C.c_int32), ("Sk", C.c_int32), ("q_offset", C.c_int64), ("k_offset", C.c_int64),
                ("causal", C.c_int32), ("scale", C.c_float), ("q_seg", C.c_int32), ("q_offset2", C.c_int64)]


class st_ring_desc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
                ("Sq", C.c_int32), ("Sk", C.c_int32), ("q_offset", C.c_int64), ("causal", C.c_int32),
                ("scale", C.c_float), ("n_chunks", C.c_int32),
                ("k_ptr", C.POINTER(C.c_void_p)), ("v_ptr", C.POINTER(C.c_void_p)),
                ("k_stride_b", C.c_int64), ("k_stride_s", C.c_int64), ("k_stride_h", C.c_int64),
                ("v_stride_b", C.c_int64), ("v_stride_s", C.c_int64), ("v_stride_h", C.c_int64),
                ("k_offset", C.POINTER(C.c_int64)), ("q_seg", C.c_int32), ("q_offset2", C.c_int64)]


class st_comm_report(C.Structure):
    _fields_ = [("ring_iterations", C.c_int32), ("startrail_iterations", C.c_int32),
                ("ring_p2p_bytes_per_iter", C.c_int64), ("startrail_p2p_bytes_per_iter", C.c_int64),
                ("ring_p2p_bytes", C.c_int64), ("startrail_p2p_bytes", C.c_int64),
                ("startrail_collective_bytes", C.c_int64), ("ring_p2p_seconds", C.c_double),
                ("startrail_p2p_seconds", C.c_double), ("startrail_collective_seconds", C.c_double)]


class st_device_report(C.Structure):
    _fields_ = [("name", C.c_char * 64), ("arch", C.c_char * 32), ("compute_units", C.c_int32), ("xcds", C.c_int32),
                ("max_clock_mhz", C.c_int32), ("memory_clock_mhz", C.c_int32), ("memory_bus_bits", C.c_int32),
                ("hbm_bytes", C.c_int64)]


class st_profile_entry(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_int32), ("total_ms", C.c_float)]


def library_path() -> str:
    return _LIB_PATH


def _load() -> C.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python paper_2407_00611_amd/build.py` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(_LIB_PATH)
    T, D, R = C.POINTER(st_tensor), C.POINTER(st_block_desc), C.POINTER(st_ring_desc)
    vp, f32p, i32p = C.c_void_p, C.c_void_p, C.POINTER(C.c_int32)
    sigs = {
        "st_attn_block_fwd": (C.c_int, [D, T, T, T, f32p, f32p, vp]),
        "st_attn_merge": (C.c_int, [f32p, f32p, f32p, f32p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp, vp]),
        "st_attn_combine": (C.c_int, [C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int32, C.c_int32, C.c_int32,
                                      C.c_int32, C.c_int32, C.c_int32, C.c_int32, f32p, f32p, C.c_int32, vp, vp]),
        "st_attn_delta": (C.c_int, [D, T, T, C.c_int32, f32p, vp]),
        "st_attn_block_bwd": (C.c_int, [D, T, T, T, T, f32p, f32p, f32p, f32p, f32p, vp, C.c_size_t, vp]),
        "st_attn_block_bwd_workspace_bytes": (C.c_size_t, [D]),
        "st_cast_from_f32": (C.c_int, [f32p, vp, C.c_int64, C.c_int32, vp]),
        "st_visit_order": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, i32p, i32p]),
        "st_team_visit_order": (C.c_int, [C.c_int32, C.c_int32, C.c_int32, i32p]),
        "st_schedule_report": (C.c_int, [C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_int64, C.c_int32,
                                         C.c_double, C.c_double, C.POINTER(st_comm_report)]),
        "st_ring_workspace_bytes": (C.c_size_t, [R, C.c_int32, C.c_int32]),
        "st_ring_fwd": (C.c_int, [R, T, i32p, i32p, C.c_int32, C.c_int32, f32p, f32p, vp, vp, C.c_size_t, vp]),
        "st_ring_bwd": (C.c_int, [R, T, T, T, C.c_int32, f32p, i32p, C.c_int32, C.c_int32, f32p,
                                  C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), vp, C.c_size_t, vp]),
        "st_ring_bwd_noalloc": (C.c_int, [R, T, T, T, C.c_int32, f32p, i32p, C.c_int32, C.c_int32, f32p,
                                          C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), vp]),
        "st_ring_bwd_noalloc_max_bytes": (C.c_size_t, []),
        "st_ring_bwd_last": (C.c_int, [R, T, T, T, C.c_int32, f32p, i32p, C.c_int32, C.c_int32, f32p,
                                       C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.c_int32,
                                       C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), vp, C.c_size_t, vp]),
        "st_device_facts": (C.c_int, [C.POINTER(st_device_report)]),
        "st_mfma_probe": (C.c_int, [vp, C.c_int64, C.c_int32, C.c_int32, f32p, C.c_int64, C.POINTER(C.c_double), vp]),
        "st_mfma_probe_mixes": (C.c_int32, []),
        "st_mfma_probe_mix_name": (C.c_char_p, [C.c_int32]),
        "st_profile_begin": (C.c_int, []),
        "st_profile_end": (C.c_int, [C.POINTER(st_profile_entry), C.c_int32, C.POINTER(C.c_int32)]),
        "st_status_str": (C.c_char_p, [C.c_int]),
        "st_last_error": (C.c_char_p, []),
        "st_version": (C.c_int32, []),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


_lib = _load()
EXPORTS = ["st_attn_block_fwd", "st_attn_merge", "st_attn_combine", "st_attn_delta", "st_attn_block_bwd", "st_attn_block_bwd_workspace_bytes", "st_cast_from_f32",
           "st_visit_order", "st_team_visit_order", "st_schedule_report", "st_ring_workspace_bytes", "st_ring_fwd", "st_ring_bwd", "st_ring_bwd_noalloc", "st_ring_bwd_noalloc_max_bytes", "st_ring_bwd_last", "st_device_facts", "st_mfma_probe", "st_mfma_probe_mixes", "st_mfma_probe_mix_name", "st_profile_begin",
           "st_profile_end", "st_status_str",
           "st_last_error", "st_version"]


def _check(status: int, where: str) -> None:
    if status != 0:
        raise StarTrailError(status, where, f"{_lib.st_status_str(status).decode()}: {_lib.st_last_error().decode()}")


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return ST_F32
    if t.dtype == torch.bfloat16:
        return ST_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _torch_dtype(code: int):
    return torch.float32 if code == ST_F32 else torch.bfloat16


def _view(t: torch.Tensor) -> st_tensor:
    if t.dim() != 4:
        raise ValueError("expected a [B, S, heads, D] tensor")
    if t.shape[3] > 1 and t.stride(3) != 1:
        raise ValueError("the D dimension must be contiguous")
    return st_tensor(t.data_ptr() if t.numel() else None, t.stride(0), t.stride(1), t.stride(2))


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _ptr(t: Optional[torch.Tensor]) -> C.c_void_p:
    return C.c_void_p(t.data_ptr() if t is not None and t.numel() else None)


def _aligned(buf: torch.Tensor, a: int) -> Tuple[int, int]:
    """First a-byte aligned address inside a byte buffer and the bytes from there to its end."""
    ptr = (buf.data_ptr() + a - 1) // a * a
    return ptr, buf.numel() * buf.element_size() - (ptr - buf.data_ptr())


def _f32_dense(t: torch.Tensor, shape, name: str) -> torch.Tensor:
    if t.dtype != torch.float32 or tuple(t.shape) != tuple(shape) or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous fp32 tensor of shape {tuple(shape)}")
    return t


def _q_runs(q_offset) -> Tuple[int, int, int]:
    """q_offset is the position of query row 0, or (position of row 0, rows in the first run, position of the
    first row of the second run) for a shard made of two runs of the sequence."""
    if isinstance(q_offset, (tuple, list)):
        off, seg, off2 = q_offset
        return int(off), int(seg), int(off2)
    return int(q_offset), 0, 0


def _block_desc(q, k, q_offset, k_offset, causal, scale) -> st_block_desc:
    B, Sq, Hq, D = q.shape
    off, seg, off2 = _q_runs(q_offset)
    return st_block_desc(_dtype_code(q), B, Hq, k.shape[2], D, Sq, k.shape[1], off, int(k_offset),
                         1 if causal else 0, float(scale), seg, off2)


def st_version() -> int:
    return int(_lib.st_version())


def st_status_str(status: int) -> str:
    return _lib.st_status_str(int(status)).decode()


def st_last_error() -> str:
    return _lib.st_last_error().decode()


def st_device_facts() -> dict:
    r = st_device_report()
    _check(_lib.st_device_facts(C.byref(r)), "st_device_facts")
    return {"name": r.name.decode(), "arch": r.arch.decode(), "compute_units": int(r.compute_units), "xcds": int(r.xcds),
            "max_clock_mhz": int(r.max_clock_mhz), "memory_clock_mhz": int(r.memory_clock_mhz),
            "memory_bus_bits": int(r.memory_bus_bits), "hbm_bytes": int(r.hbm_bytes)}


def st_mfma_probe(operands: torch.Tensor, iters: int, sink: torch.Tensor, mix: int = 0, stream=None) -> float:
    """Enqueues the MFMA loop `mix` (0: MFMAs only) on `operands` (any contiguous tensor, read as bf16 bits);
    returns the flop its MFMAs execute."""
    if not operands.is_contiguous() or sink.dtype != torch.float32 or not sink.is_contiguous():
        raise ValueError("operands must be contiguous, sink contiguous fp32")
    flop = C.c_double(0.0)
    _check(_lib.st_mfma_probe(_ptr(operands), operands.numel() * operands.element_size(), int(mix), int(iters), _ptr(sink),
                              sink.numel(), C.byref(flop), _stream(stream)), "st_mfma_probe")
    return float(flop.value)


def st_mfma_probe_mixes() -> int:
    return int(_lib.st_mfma_probe_mixes())


def st_mfma_probe_mix_name(mix: int) -> str:
    return _lib.st_mfma_probe_mix_name(int(mix)).decode()


def st_profile_begin() -> None:
    _check(_lib.st_profile_begin(), "st_profile_begin")


def st_profile_end() -> dict:
    """{kernel name: (launches, total_ms)} of everything launched since st_profile_begin()."""
    buf = (st_profile_entry * 32)()
    n = C.c_int32(0)
    _check(_lib.st_profile_end(buf, 32, C.byref(n)), "st_profile_end")
    return {buf[i].name.decode(): (int(buf[i].launches), float(buf[i].total_ms)) for i in range(n.value)}


def st_attn_block_fwd(q, k, v, q_offset: int, k_offset: int, causal: bool, scale: float,
                      o_part=None, lse_part=None, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    B, Sq, Hq, D = q.shape
    o_part = torch.empty((B, Sq, Hq, D), dtype=torch.float32, device=q.device) if o_part is None else \
        _f32_dense(o_part, (B, Sq, Hq, D), "o_part")
    lse_part = torch.empty((B, Hq, Sq), dtype=torch.float32, device=q.device) if lse_part is None else \
        _f32_dense(lse_part, (B, Hq, Sq), "lse_part")
    d = _block_desc(q, k, q_offset, k_offset, causal, scale)
    tq, tk, tv = _view(q), _view(k), _view(v)
    _check(_lib.st_attn_block_fwd(C.byref(d), C.byref(tq), C.byref(tk), C.byref(tv), _ptr(o_part), _ptr(lse_part),
                                  _stream(stream)), "st_attn_block_fwd")
    return o_part, lse_part


def st_attn_merge(o_acc, lse_acc, o_part, lse_part, out_dtype: int = ST_F32, o_out_lowp=None, stream=None) -> None:
    B, Sq, Hq, D = o_acc.shape
    _f32_dense(o_acc, (B, Sq, Hq, D), "o_acc"); _f32_dense(o_part, (B, Sq, Hq, D), "o_part")
    _f32_dense(lse_acc, (B, Hq, Sq), "lse_acc"); _f32_dense(lse_part, (B, Hq, Sq), "lse_part")
    if o_out_lowp is not None and (tuple(o_out_lowp.shape) != (B, Sq, Hq, D) or not o_out_lowp.is_contiguous()
                                   or o_out_lowp.dtype != _torch_dtype(out_dtype)):
        raise ValueError("o_out_lowp must be dense [B,Sq,Hq,D] in out_dtype")
    _check(_lib.st_attn_merge(_ptr(o_acc), _ptr(lse_acc), _ptr(o_part), _ptr(lse_part), B, Sq, Hq, D, out_dtype,
                              _ptr(o_out_lowp), _stream(stream)), "st_attn_merge")


def st_attn_combine(o_parts, lse_parts, row0: int = 0, Sq_out: int = None, out_dtype: int = ST_F32, o_out=None,
                    lse_out=None, o_out_lowp=None, stream=None):
    """n partial states of the same rows -> (o_out, lse_out) of rows [row0, row0 + Sq_out)."""
    n = len(o_parts)
    if n == 0 or len(lse_parts) != n:
        raise ValueError("need as many lse_parts as o_parts, at least one")
    B, Sq_in, Hq, D = o_parts[0].shape
    Sq_out = Sq_in - row0 if Sq_out is None else Sq_out
    for x in range(n):
        _f32_dense(o_parts[x], (B, Sq_in, Hq, D), "o_parts[x]")
        _f32_dense(lse_parts[x], (B, Hq, Sq_in), "lse_parts[x]")
    dev = o_parts[0].device
    o_out = torch.empty((B, Sq_out, Hq, D), dtype=torch.float32, device=dev) if o_out is None else \
        _f32_dense(o_out, (B, Sq_out, Hq, D), "o_out")
    lse_out = torch.empty((B, Hq, Sq_out), dtype=torch.float32, device=dev) if lse_out is None else \
        _f32_dense(lse_out, (B, Hq, Sq_out), "lse_out")
    if o_out_lowp is not None and (tuple(o_out_lowp.shape) != (B, Sq_out, Hq, D) or not o_out_lowp.is_contiguous()
                                   or o_out_lowp.dtype != _torch_dtype(out_dtype)):
        raise ValueError("o_out_lowp must be dense [B,Sq_out,Hq,D] in out_dtype")
    op = (C.c_void_p * n)(*[_ptr(t) for t in o_parts])
    lp = (C.c_void_p * n)(*[_ptr(t) for t in lse_parts])
    _check(_lib.st_attn_combine(op, lp, n, B, Sq_in, Hq, D, int(row0), int(Sq_out), _ptr(o_out), _ptr(lse_out), out_dtype,
                                _ptr(o_out_lowp), _stream(stream)), "st_attn_combine")
    return o_out, lse_out


def st_attn_delta(d_o, o, delta=None, stream=None) -> torch.Tensor:
    B, Sq, Hq, D = d_o.shape
    delta = torch.empty((B, Hq, Sq), dtype=torch.float32, device=d_o.device) if delta is None else \
        _f32_dense(delta, (B, Hq, Sq), "delta")
    d = st_block_desc(_dtype_code(d_o), B, Hq, Hq, D, Sq, 0, 0, 0, 0, 1.0)
    td, to = _view(d_o), _view(o)
    _check(_lib.st_attn_delta(C.byref(d), C.byref(td), C.byref(to), _dtype_code(o), _ptr(delta), _stream(stream)),
           "st_attn_delta")
    return delta


def st_attn_block_bwd_workspace_bytes(q, k, q_offset: int, k_offset: int, causal: bool, scale: float) -> int:
    d = _block_desc(q, k, q_offset, k_offset, causal, scale)
    return int(_lib.st_attn_block_bwd_workspace_bytes(C.byref(d)))


def st_attn_block_bwd(q, k, v, d_o, lse_final, delta, q_offset: int, k_offset: int, causal: bool, scale: float,
                      dq_acc, dk_acc, dv_acc, stream=None, workspace=None) -> None:
    """workspace: a uint8 tensor of st_attn_block_bwd_workspace_bytes(...) bytes, None to have one allocated, or
    False to pass none (the C call then keeps the dK/dV work in its general kernel)."""
    B, Sq, Hq, D = q.shape
    Sk, Hkv = k.shape[1], k.shape[2]
    _f32_dense(lse_final, (B, Hq, Sq), "lse_final"); _f32_dense(delta, (B, Hq, Sq), "delta")
    _f32_dense(dq_acc, (B, Sq, Hq, D), "dq_acc")
    _f32_dense(dk_acc, (B, Sk, Hkv, D), "dk_acc"); _f32_dense(dv_acc, (B, Sk, Hkv, D), "dv_acc")
    d = _block_desc(q, k, q_offset, k_offset, causal, scale)
    tq, tk, tv, td = _view(q), _view(k), _view(v), _view(d_o)
    need = int(_lib.st_attn_block_bwd_workspace_bytes(C.byref(d)))
    if workspace is None and need > 0:
        workspace = torch.empty(need + 256, dtype=torch.uint8, device=q.device)
    ws_ptr, ws_bytes = (None, 0) if workspace is None or workspace is False else _aligned(workspace, 256)
    _check(_lib.st_attn_block_bwd(C.byref(d), C.byref(tq), C.byref(tk), C.byref(tv), C.byref(td), _ptr(lse_final),
                                  _ptr(delta), _ptr(dq_acc), _ptr(dk_acc), _ptr(dv_acc), C.c_void_p(ws_ptr), ws_bytes,
                                  _stream(stream)),
           "st_attn_block_bwd")


def st_cast_from_f32(src, dst_dtype: int, dst=None, stream=None) -> torch.Tensor:
    if src.dtype != torch.float32 or not src.is_contiguous():
        raise ValueError("src must be contiguous fp32")
    dst = torch.empty(src.shape, dtype=_torch_dtype(dst_dtype), device=src.device) if dst is None else dst
    if not dst.is_contiguous() or dst.numel() != src.numel() or dst.dtype != _torch_dtype(dst_dtype):
        raise ValueError("dst must be contiguous, of dst_dtype and as large as src")
    _check(_lib.st_cast_from_f32(_ptr(src), _ptr(dst), src.numel(), dst_dtype, _stream(stream)), "st_cast_from_f32")
    return dst


def st_team_visit_order(P: int, Cteam: int, rank: int) -> List[int]:
    out = (C.c_int32 * max(int(P), 1))()              # the library validates the layout; P entries always suffice
    _check(_lib.st_team_visit_order(int(P), int(Cteam), int(rank), out), "st_team_visit_order")
    return list(out)[:int(P) // (int(Cteam) * int(Cteam))]


def st_schedule_report(P: int, Cteam: int, B: int, N: int, H: int, bytes_per_element: int = 2,
                       W: float = 1.0, L: float = 0.0) -> dict:
    out = st_comm_report()
    _check(_lib.st_schedule_report(int(P), int(Cteam), int(B), int(N), int(H), int(bytes_per_element), float(W), float(L),
                                   C.byref(out)), "st_schedule_report")
    return {name: getattr(out, name) for name, _ in st_comm_report._fields_}


def st_visit_order(P: int, Cteam: int, rank: int) -> Tuple[List[int], List[int]]:
    n = max(int(P), 1)
    shard = (C.c_int32 * n)()
    member = (C.c_int32 * n)()
    _check(_lib.st_visit_order(int(P), int(Cteam), int(rank), shard, member), "st_visit_order")
    return list(shard), list(member)


class _Ring:
    """Keeps the host-side tables of an st_ring_desc alive for the duration of a call."""

    def __init__(self, q, k_chunks: Sequence[torch.Tensor], v_chunks: Sequence[torch.Tensor], q_offset: int,
                 k_offsets: Sequence[int], causal: bool, scale: float):
        n = len(k_chunks)
        if n < 1 or len(v_chunks) != n or len(k_offsets) != n:
            raise ValueError("need one K, one V and one offset per chunk")
        B, Sq, Hq, D = q.shape
        k0, v0 = k_chunks[0], v_chunks[0]
        for k, v in zip(k_chunks, v_chunks):
            if k.shape != k0.shape or v.shape != k0.shape or k.stride() != k0.stride() or v.stride() != v0.stride() \
                    or k.dtype != q.dtype or v.dtype != q.dtype:
                raise ValueError("all chunks must share shape, strides and dtype")
            _view(k), _view(v)
        self.k_ptr = (C.c_void_p * n)(*[k.data_ptr() for k in k_chunks])
        self.v_ptr = (C.c_void_p * n)(*[v.data_ptr() for v in v_chunks])
        self.k_off = (C.c_int64 * n)(*[int(x) for x in k_offsets])
        off, seg, off2 = _q_runs(q_offset)
        self.desc = st_ring_desc(_dtype_code(q), B, Hq, k0.shape[2], D, Sq, k0.shape[1], off,
                                 1 if causal else 0, float(scale), n,
                                 C.cast(self.k_ptr, C.POINTER(C.c_void_p)), C.cast(self.v_ptr, C.POINTER(C.c_void_p)),
                                 k0.stride(0), k0.stride(1), k0.stride(2), v0.stride(0), v0.stride(1), v0.stride(2),
                                 C.cast(self.k_off, C.POINTER(C.c_int64)), seg, off2)


def st_ring_workspace_bytes(q, k_chunks, v_chunks, q_offset, k_offsets, causal, scale, mode: int,
                            backward: bool) -> int:
    r = _Ring(q, k_chunks, v_chunks, q_offset, k_offsets, causal, scale)
    return int(_lib.st_ring_workspace_bytes(C.byref(r.desc), mode, 1 if backward else 0))


def _i32_array(xs: Optional[Sequence[int]]):
    if xs is None:
        return None
    return (C.c_int32 * max(len(xs), 1))(*[int(x) for x in xs])


def st_ring_fwd(q, k_chunks, v_chunks, q_offset: int, k_offsets: Sequence[int], causal: bool, scale: float,
                order: Sequence[int], member_of: Optional[Sequence[int]] = None, mode: int = ST_RING_FUSED,
                o_acc=None, lse=None, o_lowp=None, want_lowp: bool = True, workspace=None, stream=None):
    """Returns (o_acc fp32, lse fp32, o_lowp or None)."""
    B, Sq, Hq, D = q.shape
    r = _Ring(q, k_chunks, v_chunks, q_offset, k_offsets, causal, scale)
    o_acc = torch.empty((B, Sq, Hq, D), dtype=torch.float32, device=q.device) if o_acc is None else \
        _f32_dense(o_acc, (B, Sq, Hq, D), "o_acc")
    lse = torch.empty((B, Hq, Sq), dtype=torch.float32, device=q.device) if lse is None else \
        _f32_dense(lse, (B, Hq, Sq), "lse")
    if o_lowp is None and want_lowp:
        o_lowp = torch.empty((B, Sq, Hq, D), dtype=q.dtype, device=q.device)
    need = int(_lib.st_ring_workspace_bytes(C.byref(r.desc), mode, 0))
    if workspace is None:
        workspace = torch.empty(need + 256, dtype=torch.uint8, device=q.device)
    ws_ptr = (workspace.data_ptr() + 255) // 256 * 256
    ws_bytes = workspace.numel() * workspace.element_size() - (ws_ptr - workspace.data_ptr())
    tq = _view(q)
    _check(_lib.st_ring_fwd(C.byref(r.desc), C.byref(tq), _i32_array(order), _i32_array(member_of), len(order), mode,
                            _ptr(o_acc), _ptr(lse), _ptr(o_lowp), C.c_void_p(ws_ptr), ws_bytes, _stream(stream)),
           "st_ring_fwd")
    return o_acc, lse, o_lowp


def st_ring_bwd(q, k_chunks, v_chunks, d_o, o, lse_final, q_offset: int, k_offsets: Sequence[int], causal: bool,
                scale: float, order: Sequence[int], dq_acc, dk_acc: Sequence[Optional[torch.Tensor]],
                dv_acc: Sequence[Optional[torch.Tensor]], mode: int = ST_RING_FUSED, workspace=None,
                stream=None) -> None:
    B, Sq, Hq, D = q.shape
    r = _Ring(q, k_chunks, v_chunks, q_offset, k_offsets, causal, scale)
    n = len(k_chunks)
    _f32_dense(dq_acc, (B, Sq, Hq, D), "dq_acc"); _f32_dense(lse_final, (B, Hq, Sq), "lse_final")
    kv_shape = tuple(k_chunks[0].shape)
    for t in list(dk_acc) + list(dv_acc):
        if t is not None:
            _f32_dense(t, kv_shape, "dk_acc/dv_acc entry")
    dk_ptr = (C.c_void_p * n)(*[(t.data_ptr() if t is not None else None) for t in dk_acc])
    dv_ptr = (C.c_void_p * n)(*[(t.data_ptr() if t is not None else None) for t in dv_acc])
    need = int(_lib.st_ring_workspace_bytes(C.byref(r.desc), mode, 1))
    if workspace is None:
        workspace = torch.empty(need + 256, dtype=torch.uint8, device=q.device)
    ws_ptr = (workspace.data_ptr() + 255) // 256 * 256
    ws_bytes = workspace.numel() * workspace.element_size() - (ws_ptr - workspace.data_ptr())
    tq, td, to = _view(q), _view(d_o), _view(o)
    _check(_lib.st_ring_bwd(C.byref(r.desc), C.byref(tq), C.byref(td), C.byref(to), _dtype_code(o), _ptr(lse_final),
                            _i32_array(order), len(order), mode, _ptr(dq_acc),
                            C.cast(dk_ptr, C.POINTER(C.c_void_p)), C.cast(dv_ptr, C.POINTER(C.c_void_p)),
                            C.c_void_p(ws_ptr), ws_bytes, _stream(stream)), "st_ring_bwd")


def st_ring_bwd_noalloc_max_bytes() -> int:
    return int(_lib.st_ring_bwd_noalloc_max_bytes())


def st_ring_bwd_noalloc(q, k_chunks, v_chunks, d_o, o, lse_final, q_offset: int, k_offsets: Sequence[int], causal: bool,
                        scale: float, order: Sequence[int], dq_acc, dk_acc: Sequence[Optional[torch.Tensor]],
                        dv_acc: Sequence[Optional[torch.Tensor]], mode: int = ST_RING_FUSED, stream=None) -> None:
    """st_ring_bwd on the library's static scratch: this wrapper allocates no device memory either."""
    B, Sq, Hq, D = q.shape
    r = _Ring(q, k_chunks, v_chunks, q_offset, k_offsets, causal, scale)
    n = len(k_chunks)
    _f32_dense(dq_acc, (B, Sq, Hq, D), "dq_acc"); _f32_dense(lse_final, (B, Hq, Sq), "lse_final")
    kv_shape = tuple(k_chunks[0].shape)
    for t in list(dk_acc) + list(dv_acc):
        if t is not None:
            _f32_dense(t, kv_shape, "dk_acc/dv_acc entry")
    dk_ptr = (C.c_void_p * n)(*[(t.data_ptr() if t is not None else None) for t in dk_acc])
    dv_ptr = (C.c_void_p * n)(*[(t.data_ptr() if t is not None else None) for t in dv_acc])
    tq, td, to = _view(q), _view(d_o), _view(o)
    _check(_lib.st_ring_bwd_noalloc(C.byref(r.desc), C.byref(tq), C.byref(td), C.byref(to), _dtype_code(o),
                                    _ptr(lse_final), _i32_array(order), len(order), mode, _ptr(dq_acc),
                                    C.cast(dk_ptr, C.POINTER(C.c_void_p)), C.cast(dv_ptr, C.POINTER(C.c_void_p)),
                                    _stream(stream)), "st_ring_bwd_noalloc")


def st_ring_bwd_last(q, k_chunks, v_chunks, d_o, o, lse_final, q_offset: int, k_offsets: Sequence[int], causal: bool,
                     scale: float, order: Sequence[int], dq_acc, dk_acc: Sequence[Optional[torch.Tensor]],
                     dv_acc: Sequence[Optional[torch.Tensor]], assign: bool = False,
                     dk_lowp: Optional[Sequence[Optional[torch.Tensor]]] = None,
                     dv_lowp: Optional[Sequence[Optional[torch.Tensor]]] = None, mode: int = ST_RING_FUSED,
                     workspace=None, stream=None) -> None:
    B, Sq, Hq, D = q.shape
    r = _Ring(q, k_chunks, v_chunks, q_offset, k_offsets, causal, scale)
    n = len(k_chunks)
    _f32_dense(dq_acc, (B, Sq, Hq, D), "dq_acc"); _f32_dense(lse_final, (B, Hq, Sq), "lse_final")
    kv_shape = tuple(k_chunks[0].shape)
    for t in list(dk_acc) + list(dv_acc):
        if t is not None:
            _f32_dense(t, kv_shape, "dk_acc/dv_acc entry")

    def table(ts):
        if ts is None:
            return None
        for t in ts:
            if t is not None and not (t.is_cuda and t.is_contiguous() and t.dtype == q.dtype and tuple(t.shape) == kv_shape):
                raise ValueError("dk_lowp/dv_lowp entry: expected a dense device tensor shaped like a chunk, in the dtype of q")
        return (C.c_void_p * n)(*[(t.data_ptr() if t is not None else None) for t in ts])

    dk_ptr, dv_ptr = _ptr_table(dk_acc, n), _ptr_table(dv_acc, n)
    lk, lv = table(dk_lowp), table(dv_lowp)
    need = int(_lib.st_ring_workspace_bytes(C.byref(r.desc), mode, 1))
    if workspace is None:
        workspace = torch.empty(need + 256, dtype=torch.uint8, device=q.device)
    ws_ptr = (workspace.data_ptr() + 255) // 256 * 256
    ws_bytes = workspace.numel() * workspace.element_size() - (ws_ptr - workspace.data_ptr())
    tq, td, to = _view(q), _view(d_o), _view(o)
    vpp = C.POINTER(C.c_void_p)
    _check(_lib.st_ring_bwd_last(C.byref(r.desc), C.byref(tq), C.byref(td), C.byref(to), _dtype_code(o), _ptr(lse_final),
                                 _i32_array(order), len(order), mode, _ptr(dq_acc), C.cast(dk_ptr, vpp), C.cast(dv_ptr, vpp),
                                 ST_KV_ASSIGN if assign else 0, C.cast(lk, vpp) if lk is not None else None,
                                 C.cast(lv, vpp) if lv is not None else None,
                                 C.c_void_p(ws_ptr), ws_bytes, _stream(stream)), "st_ring_bwd_last")


def _ptr_table(ts, n):
    return (C.c_void_p * n)(*[(t.data_ptr() if t is not None else None) for t in ts])
