"""Seeded synthetic inputs for the ring-attention share workloads.

This module only *produces data*: shapes, global token offsets, seeded normal
values and their rounding to the storage dtype.  It contains none of the
attention arithmetic and is imported by the tests and the benchmark to feed
both the HIP path and the CPU oracle with the same bytes.

Workloads are stand-ins shaped like the paper's runs (Section 4 setup: batch 1,
bf16, GPT-7B-like 32 heads x 128, sequences of 64K-512K tokens split over a
ring of P GPUs); the paper's models, weights and datasets are not used.

Values: i.i.d. N(0, sigma) drawn in fp32 from a Philox counter-based generator
keyed by ``1000 * cfg + tensor_id`` (Q=0, dO=3) and, for the KV chunks,
``1000 * cfg + 100 * tensor_id + 10_000 * (chunk + 1)`` (K=1, V=2), then rounded
to the storage dtype (bf16 round-to-nearest-even, or kept as fp32).
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

TENSOR_Q, TENSOR_K, TENSOR_V, TENSOR_DO = 0, 1, 2, 3


@dataclass(frozen=True)
class Workload:
    """One GPU's share of ring attention: a resident Q shard and n KV chunks."""

    name: str
    cfg: int                 # seed family
    dtype: str               # "f32" or "bf16" (storage dtype of Q, K, V, dO)
    B: int
    Hq: int
    Hkv: int
    D: int
    Sq: int                  # tokens in the Q shard
    Sk: int                  # tokens per KV chunk
    n_chunks: int
    q_offset: int            # global position of Q row 0
    causal: bool
    backward: bool
    sigma: float = 1.0
    ring_P: int = 0          # ring size for the visit order (0: natural order)
    ring_C: int = 1          # team size of the concentric layout
    ring_rank: int = 0
    k_ramp: float = 0.0      # K chunk j is scaled by 1 + k_ramp * j: later chunks raise the row maxima sharply
    q_seg: int = 0           # > 0: query rows [q_seg, Sq) are a second run of the sequence that starts at q_offset2
    q_offset2: int = 0

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.D))

    @property
    def N(self) -> int:
        return self.Sk * self.n_chunks

    def k_offset(self, j: int) -> int:
        return j * self.Sk

    def q_positions(self) -> np.ndarray:
        """Global position of every query row."""
        i = np.arange(self.Sq, dtype=np.int64)
        if self.q_seg > 0:
            return np.where(i < self.q_seg, self.q_offset + i, self.q_offset2 + i - self.q_seg)
        return self.q_offset + i

    @property
    def q_where(self):
        """The shard's placement as the binding takes it: a position, or (position, rows, position) for two runs."""
        return (self.q_offset, self.q_seg, self.q_offset2) if self.q_seg > 0 else self.q_offset


def paper_workloads() -> List[Workload]:
    """The five benchmark configurations (index 0..4 = config 1..5)."""
    return [
        Workload("cfg1_tiny_f32", 1, "f32", 1, 1, 1, 64, 128, 128, 4, 0, False, True),
        Workload("cfg2_bf16_fwd", 2, "bf16", 1, 8, 8, 128, 1024, 1024, 8, 3072, True, False,
                 ring_P=8, ring_C=1, ring_rank=3),
        Workload("cfg3_bf16_ring16", 3, "bf16", 1, 32, 32, 128, 2048, 2048, 16, 32768 - 2048,
                 True, True, ring_P=16, ring_C=1, ring_rank=15),
        Workload("cfg4_gqa_concentric_4x8", 4, "bf16", 1, 32, 8, 128, 4096, 4096, 32,
                 131072 - 4096, True, True, ring_P=32, ring_C=4, ring_rank=31),
        Workload("cfg5_long_context", 5, "bf16", 1, 16, 16, 128, 8192, 8192, 64,
                 524288 - 8192, True, True, sigma=0.5, ring_P=64, ring_C=1, ring_rank=63),
    ]


def team_workload() -> Workload:
    """The model and layout of configuration 4 (GQA 32/8 heads, D = 128, 131072 tokens, P = 32 GPUs in teams
    of C = 4) in the shape one GPU really sees in the concentric layout: the resident queries are the whole
    team's C N/P = 16384 rows (last team), the keys / values are the P/C = 8 gathered team buffers of 16384
    tokens, of which a GPU meets P/C^2 = 2."""
    return Workload("team4x8_gqa_gathered", 6, "bf16", 1, 32, 8, 128, 16384, 16384, 8, 131072 - 16384, True, True,
                    ring_P=32, ring_C=4, ring_rank=31)


def dit_workload() -> Workload:
    """A share shaped like the paper's diffusion-transformer runs (model table: DiT 1B, 24 heads, hidden 1536,
    i.e. head size 64; full mask; scaling runs at 128K tokens on 8 GPUs): rank 3 of a ring of 8, 16384-token
    shard, 8 chunks of 16384 tokens, non-causal, bf16."""
    return Workload("dit1b_full_mask_ring8", 7, "bf16", 1, 24, 24, 64, 16384, 16384, 8, 3 * 16384, False, True,
                    ring_P=8, ring_C=1, ring_rank=3)


def zigzag_workload(rank: int = 0) -> Workload:
    """The model of configuration 4 under the load-balanced causal placement (appendix "Sequence Parallelism
    Dataloader"): the sequence of 131072 tokens is cut into 2 P = 64 pieces of 2048 tokens and rank r of the
    ring of P = 32 holds pieces r and 2 P - 1 - r.  Query shard: those two pieces (4096 rows in two runs); the
    ring delivers every rank's two pieces, here 64 chunks of 2048 tokens."""
    P, m = 32, 2048
    return Workload(f"zigzag32_gqa_rank{rank}", 8, "bf16", 1, 32, 8, 128, 2 * m, m, 2 * P, rank * m, True, True,
                    ring_P=P, ring_C=1, ring_rank=rank, q_seg=m, q_offset2=(2 * P - 1 - rank) * m)


def small_workload(name="small", dtype="bf16", B=1, Hq=2, Hkv=1, D=128, Sq=192, Sk=160,
                   n_chunks=3, q_offset=None, causal=True, cfg=90, sigma=1.0) -> Workload:
    """A ragged multi-tile case the oracle finishes in well under a second."""
    if q_offset is None:
        q_offset = Sk * n_chunks - Sq if causal else 0
    return Workload(name, cfg, dtype, B, Hq, Hkv, D, Sq, Sk, n_chunks, q_offset, causal, True,
                    sigma=sigma)


# --------------------------------------------------------------------------
# value generation and storage rounding
# --------------------------------------------------------------------------

def normal_f32(seed: int, shape, sigma: float = 1.0) -> np.ndarray:
    """i.i.d. N(0, sigma^2) fp32 values from a Philox stream keyed by ``seed``."""
    gen = np.random.Generator(np.random.Philox(key=int(seed)))
    x = gen.standard_normal(size=shape, dtype=np.float32)
    if sigma != 1.0:
        x *= np.float32(sigma)
    return x


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); returns the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 exactly."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Inputs:
    """Storage-exact inputs.  ``*_f32`` hold the storage values widened to fp32;
    ``*_bits`` (bf16 only) hold the 16-bit patterns that go to the GPU."""

    w: Workload
    q: np.ndarray                      # [B,Sq,Hq,D] fp32
    k: List[np.ndarray]                # n x [B,Sk,Hkv,D] fp32
    v: List[np.ndarray]
    d_o: Optional[np.ndarray]          # [B,Sq,Hq,D] fp32 or None
    q_bits: Optional[np.ndarray] = None
    k_bits: List[np.ndarray] = field(default_factory=list)
    v_bits: List[np.ndarray] = field(default_factory=list)
    d_o_bits: Optional[np.ndarray] = None


def _store(x: np.ndarray, dtype: str):
    if dtype == "bf16":
        bits = f32_to_bf16_bits(x)
        return bf16_bits_to_f32(bits), bits
    return x, None


def chunk_seed(cfg: int, tensor_id: int, chunk: int) -> int:
    return 1000 * cfg + 100 * tensor_id + 10_000 * (chunk + 1)


def make_chunk(w: Workload, tensor_id: int, j: int, keep_f32: bool = True):
    """K (tensor_id=1) or V (2) chunk j: (fp32 storage-exact values or None, bits or None)."""
    sigma = w.sigma * (1.0 + w.k_ramp * j) if tensor_id == TENSOR_K else w.sigma
    x = normal_f32(chunk_seed(w.cfg, tensor_id, j), (w.B, w.Sk, w.Hkv, w.D), sigma)
    f, bits = _store(x, w.dtype)
    return (f if keep_f32 or bits is None else None), bits


def make_inputs(w: Workload, threads: int = 8, keep_f32: bool = True) -> Inputs:
    """All tensors of a workload.  ``keep_f32=False`` drops the widened fp32
    copies of bf16 KV chunks (the big configurations regenerate slices on demand)."""
    q, q_bits = _store(normal_f32(1000 * w.cfg + TENSOR_Q, (w.B, w.Sq, w.Hq, w.D), w.sigma), w.dtype)
    d_o = d_o_bits = None
    if w.backward:
        d_o, d_o_bits = _store(normal_f32(1000 * w.cfg + TENSOR_DO, (w.B, w.Sq, w.Hq, w.D), w.sigma),
                               w.dtype)
    jobs = [(t, j) for j in range(w.n_chunks) for t in (TENSOR_K, TENSOR_V)]
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        res = list(ex.map(lambda tj: make_chunk(w, tj[0], tj[1], keep_f32), jobs))
    k = [res[2 * j][0] for j in range(w.n_chunks)]
    v = [res[2 * j + 1][0] for j in range(w.n_chunks)]
    k_bits = [res[2 * j][1] for j in range(w.n_chunks)]
    v_bits = [res[2 * j + 1][1] for j in range(w.n_chunks)]
    return Inputs(w, q, k, v, d_o, q_bits, k_bits, v_bits, d_o_bits)


def sampled_rows(w: Workload, head: int, count: int = 256) -> np.ndarray:
    """Sorted distinct query-row indices of the shard sampled for ``head``
    (seed 5000 + head).  The first and last rows are always included."""
    gen = np.random.Generator(np.random.Philox(key=5000 + int(head)))
    count = min(count, w.Sq)
    rows = gen.choice(w.Sq, size=count, replace=False)
    rows[0], rows[-1] = 0, w.Sq - 1
    return np.unique(rows).astype(np.int64)


def visible_pairs(w: Workload, chunks: Optional[Sequence[int]] = None) -> int:
    """Exact number of (query, key) pairs per head that the mask leaves visible, over all chunks or
    over the listed ones."""
    chunks = range(w.n_chunks) if chunks is None else chunks
    if not w.causal:
        return w.Sq * w.Sk * len(chunks)
    i = w.q_positions()
    return int(sum(np.clip(i - w.k_offset(j) + 1, 0, w.Sk).sum() for j in chunks))


def algorithmic_flop(w: Workload, chunks: Optional[Sequence[int]] = None):
    """(fwd, bwd) FLOP: two contractions forward and five backward over visible pairs."""
    pairs = visible_pairs(w, chunks) * w.Hq * w.B
    return 4 * w.D * pairs, (10 * w.D * pairs if w.backward else 0)
