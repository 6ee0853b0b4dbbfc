#!/usr/bin/env python3
"""Generates the gfx950 assembly of the dQ main loop (head_dim 128, or 64) as a C string literal.

    python gen_bwd_dq_asm.py > st_bwd_dq_asm.inc          (build.py does this before compiling)
    python gen_bwd_dq_asm.py 64 > st_bwd_dq64_asm.inc     (head_dim 64: half the MFMAs per group, 128-byte tile rows)

Body of ONE `asm volatile` statement in st_bwd_dq_fast.hip.  A workgroup (4 wavefronts) owns 256 queries
of one head, 64 per wavefront as two 32-query blocks, and walks the 64-key tiles that every one of its
rows sees in full (tiles that need a mask, ragged tails and ragged query tiles go to the general kernel).
The MFMA C layout is "lane = query column", so lse and Delta are one register per lane and block.
Q and dO fragments stay in AGPRs (MFMA B operands may come from there), the dQ^T accumulators too.
The Q fragments are multiplied by scale * log2(e) once (and rounded to bf16 again) and the S^T accumulators
start from -lse * log2(e), the dP'^T accumulators from -Delta: the MFMAs deliver the exponent of P and
dP - Delta directly.

Per 32-key block i and wavefront, three groups of 16 MFMAs, software-pipelined across blocks so that
every VALU result is needed one group later than it is produced:
    group A   S^T(i+1)  = K Q^T                  A: K rows of block i+1 from LDS        VALU: dS(i) = P(i) dP'(i), bf16 pack
    group B   dQ^T     += K^T dS^T(i)            A: K^T of block i by transpose reads   VALU: P(i+1) = exp2(S c - lse log2e)
    group C   dP'^T(i+1) = V dO^T - Delta        A: V rows of block i+1, C init: -Delta VALU: rest of P(i+1)
K / V tiles (64 keys) arrive by direct global->LDS loads into a 4-stage ring, three tiles ahead; one
barrier per tile.  The chunk table (base pointers, tiles per chunk) sits in LDS, written by the C++ side.
"""
import os
import sys

from st_asmgen import Emitter, ar, sr, vr, write_inc

D = 64 if "64" in sys.argv[1:] else 128              # head_dim
KS, DB, QB, NS = D // 16, D // 32, 2, 4
ROW = 2 * D                                          # bytes of one K / V row in LDS
TILE = 64 * ROW                                      # one 64-key tile
NDMA = TILE // 4096                                  # direct-to-LDS loads per wavefront and tile (4 wavefronts x 1 KiB each)
NA, NB, NC = 2 * KS, 4 * DB, 2 * KS                  # MFMAs of the three groups of a key block
NSLOT = NA + NB + NC
SPLIT = 4 * 2 * TILE > 65536                         # ring beyond the 16-bit offset field: second set of base registers

# ---- AGPRs
def ACC(db, qb): return 16 * (2 * db + qb)
def QF(qb, ks): return 128 + 4 * (KS * qb + ks)
def DOF(qb, ks): return 192 + 4 * (KS * qb + ks)

# ---- VGPRs
def SBUF(buf, qb): return 32 * buf + 16 * qb        # two score buffers (later P, fp32)
def DP(qb): return 64 + 16 * qb                     # dP', later dS, later packed dS in [4m .. 4m+3]
def ND(qb): return 96 + 16 * qb                     # sixteen copies of -Delta (MFMA C operand)
def NL(qb): return 128 + 16 * qb                    # sixteen copies of -lse * log2(e) (MFMA C operand)
POOL0 = 160                                          # 3 rings x 4 fragments x 4 registers
TMP = 208                                            # 208..214
DQOFF = 215
XL, XH = 216, 224                                    # natural-read offsets: stages 0-1 / stages 2-3
TRLO_L, TRHI_L, TRLO_H, TRHI_H = 232, 236, 240, 244
KOFF, VOFF = 248, 252                                # per-lane global offsets of the 4 DMA instructions per tensor
# inputs (pinned by the C++ side) sit in the fragment pool, which the prologue does not use
IN_VA, IN_VB = 160, 176                              # v[160:175], v[176:179]
I_QROW0, I_QROW1, I_DOROW0, I_DOROW1 = 160, 162, 164, 166
I_NL0, I_NL1, I_ND0, I_ND1, I_XBASE, I_GF16, I_TRBASE, I_LF16 = 168, 169, 170, 171, 172, 173, 174, 175
I_KOFF0, I_VOFF0, I_DQOFF = 176, 177, 178
PT = 184                                             # 184..199: temporaries of the prologue
(S_LDS, S_WAVE, S_NT, S_KRS16, S_VRS16, S_SCALE, S_DQPTR, S_DQQB, S_TBL, S_KTILE, S_VTILE) = (32, 33, 34, 35, 36, 37, 38, 40, 41, 42, 43)
# scalar temporaries
S_CEXP, T_M0, T_REM, D_KPTR, D_VPTR, D_LEFT, D_IDX, D_TBL, T_X = 47, 64, 65, 66, 68, 70, 71, 72, 73

# ---- LDS map
def KT(s): return 2 * TILE * s
def VT(s): return 2 * TILE * s + TILE
TBL = 2 * TILE * NS                                     # 64 entries x 32 bytes: k lo/hi, v lo/hi, tiles, pad
LDS_BYTES = TBL + 2048

LAT = int(os.environ.get("ST_GEN_DQ_LAT", 3))
BUDGET = int(os.environ.get("ST_GEN_DQ_BUDGET", 5 if D == 128 else 7))


class Pipe:
    """Emits blocks one after the other; LDS reads wanted before a block's first MFMA are issued at the
    tail of the block before it."""

    def __init__(self, e):
        self.e = e
        self.frag_reg = {}
        self.uses_left = {}
        self.owner = {}
        self.pending_valu = []     # VALU-1 items may not spill across blocks; checked at block end

    def alloc(self, ring, idx, tag, uses):
        slot = 4 * ring + idx % 4
        old = self.owner.get(slot)
        assert old is None or self.uses_left[old] == 0, f"fragment {old} overwritten by {tag} before its last use"
        self.owner[slot] = tag
        self.uses_left[tag] = uses
        self.frag_reg[tag] = POOL0 + 4 * slot
        return POOL0 + 4 * slot

    def use(self, tag):
        assert self.uses_left[tag] > 0, tag
        self.uses_left[tag] -= 1
        return self.frag_reg[tag]


def upper(stage): return SPLIT and stage >= 2
def xreg(stage, ks): return (XH if upper(stage) else XL) + ks
def trregs(stage, db): return ((TRLO_H, TRHI_H) if upper(stage) else (TRLO_L, TRHI_L))
def imm(stage, tensor_base): return tensor_base - (65536 if upper(stage) else 0)


def read_k(p, stage, kb, ks, seq):
    """K rows of block (stage, kb), contraction step ks: A operand of S^T."""
    tag = f"k{seq}_{ks}"
    r = p.alloc(0, ks, tag, QB)
    p.e.ds_read(f"ds_read_b128 {vr(r, 4)}, {vr(xreg(stage, ks))} offset:{imm(stage, KT(stage)) + 32 * ROW * kb}", tag)


def read_v(p, stage, kb, ks, seq):
    tag = f"v{seq}_{ks}"
    r = p.alloc(2, ks, tag, QB)
    p.e.ds_read(f"ds_read_b128 {vr(r, 4)}, {vr(xreg(stage, ks))} offset:{imm(stage, VT(stage)) + 32 * ROW * kb}", tag)


def read_kt(p, stage, kb, m, db, seq):
    """K^T fragment (32 d rows x 16 keys) of block (stage, kb): A operand of dQ^T."""
    tag = f"t{seq}_{m}_{db}"
    r = p.alloc(1, DB * m + db, tag, QB)
    lo, hi = trregs(stage, db)
    off = imm(stage, KT(stage)) + 32 * ROW * kb + 16 * ROW * m
    p.e.ds_read(f"ds_read_b64_tr_b16 {vr(r, 2)}, {vr(lo + db)} offset:{off}", tag + "lo")
    p.e.ds_read(f"ds_read_b64_tr_b16 {vr(r + 2, 2)}, {vr(hi + db)} offset:{off}", tag)


def gen_block(p, cur, nxt, nxt2, pbuf, seq, do_b=True, do_ac=True, head=None, prefetched=True, side=None):
    """cur / nxt / nxt2 = (stage, kb) of blocks i, i+1, i+2 (nxt2 only for the prefetch at the tail).
    pbuf = score buffer that holds P(i); S(i+1) goes to the other one.  `head` is emitted in front of the
    first MFMA (barrier and DMA of a new tile).  seq numbers the block for fragment tags: tags of block
    seq + 1's first reads are created here, so that the next block finds them."""
    e = p.e
    nbuf = 1 - pbuf
    e.comment(f"======== block {cur}: S^T{nxt} -> buffer {nbuf} | dQ^T += K^T dS^T{cur} | dP'^T{nxt}")
    slots = []
    reads = {k: [] for k in range(-1, NSLOT)}

    def plan(first_use, fn):
        reads[max(first_use - LAT, -1)].append(fn)

    if do_ac:
        for ks in range(KS):
            if not (prefetched and ks < 2):                    # ks 0, 1 were requested at the tail of the block before
                plan(2 * ks, (lambda ks=ks: read_k(p, nxt[0], nxt[1], ks, seq)))
            for qb in range(QB):
                slots.append(("A", ks, qb))
    else:
        slots += [None] * NA
    if do_b:
        for m in range(2):
            for db in range(DB):
                plan(NA + 2 * (DB * m + db), (lambda m=m, db=db: read_kt(p, cur[0], cur[1], m, db, seq)))
                for qb in range(QB):
                    slots.append(("B", m, db, qb))
    else:
        slots += [None] * NB
    if do_ac:
        for ks in range(KS):
            plan(NA + NB + 2 * ks, (lambda ks=ks: read_v(p, nxt[0], nxt[1], ks, seq)))
            for qb in range(QB):
                slots.append(("C", ks, qb))
        if nxt2 is not None:
            for ks in range(2):
                reads[NSLOT - 4 + ks].append(lambda ks=ks: read_k(p, nxt2[0], nxt2[1], ks, seq + 1))
    else:
        slots += [None] * NC

    # ---- VALU work: (earliest slot, text, registers written, issue units)
    valu = []
    if do_b:   # dS(i) = P(i) dP'(i), packed in place; dP'(i) was written by the last group of the block before
        for m in range(2):
            for qb in range(QB):
                for v in range(8 * m, 8 * m + 8):
                    valu.append((2 + qb, f"v_mul_f32 {vr(DP(qb) + v)}, {vr(SBUF(pbuf, qb) + v)}, {vr(DP(qb) + v)}", (), 1))
                for i in range(4):
                    d, a = DP(qb) + 4 * m + i, DP(qb) + 8 * m + 2 * i
                    valu.append((2 + qb, f"v_cvt_pk_bf16_f32 {vr(d)}, {vr(a)}, {vr(a + 1)}", (d,), 1))
    # the first VALU reader of an MFMA result comes three MFMA issues after the MFMA
    early1 = NA + 1 if do_b else NA + NB + 2
    if do_ac:  # P(i+1) = exp2(exponent); S^T(i+1)[qb] is written by slot NA - 2 + qb
        for qb in range(QB):
            for grp in range(4):
                vs = [SBUF(nbuf, qb) + 4 * grp + i for i in range(4)]
                for r in vs:
                    valu.append((early1 + qb, f"v_exp_f32 {vr(r)}, {vr(r)}", (), 2))
    vi = [0]
    produced = {}

    def emit_valu(item):
        e.valu(item[1], item[2])
        for r in item[2]:
            produced[r] = True
        return item[3]

    if head is not None:
        head()
    for fn in reads[-1]:
        fn()
    for k, sl in enumerate(slots):
        if sl is None:
            for fn in reads[k]:
                fn()
            continue
        if sl[0] == "A":
            _, ks, qb = sl
            tag = f"k{seq}_{ks}"
            e.need(tag)
            d = vr(SBUF(nbuf, qb), 16)
            e.mfma(d, vr(p.use(tag), 4), ar(QF(qb, ks), 4), vr(NL(qb), 16) if ks == 0 else d)
        elif sl[0] == "B":
            _, m, db, qb = sl
            tag = f"t{seq}_{m}_{db}"
            e.need(tag)
            b0 = DP(qb) + 4 * m
            while not all(produced.get(b0 + i) for i in range(4)):
                emit_valu(valu[vi[0]])
                vi[0] += 1
            acc = ar(ACC(db, qb), 16)
            e.mfma(acc, vr(p.use(tag), 4), vr(b0, 4), acc, breads=[b0 + i for i in range(4)])
        else:
            _, ks, qb = sl
            tag = f"v{seq}_{ks}"
            e.need(tag)
            d = vr(DP(qb), 16)
            e.mfma(d, vr(p.use(tag), 4), ar(DOF(qb, ks), 4), vr(ND(qb), 16) if ks == 0 else d)
        units = 0
        for fn in reads[k]:
            n0 = len(e.ds)
            fn()
            units += len(e.ds) - n0
        if side and k in side:                           # tile request / stream bookkeeping spread under the MFMAs
            for ln in side[k]:
                e.raw(ln)
            units += 2
        while vi[0] < len(valu) and valu[vi[0]][0] <= k and units + valu[vi[0]][3] <= BUDGET:
            units += emit_valu(valu[vi[0]])
            vi[0] += 1
    if not do_b:                     # pipeline fill: fewer slots to hide the exponentials under
        while vi[0] < len(valu):
            emit_valu(valu[vi[0]])
            vi[0] += 1
    assert vi[0] == len(valu), f"VALU work left over: {len(valu) - vi[0]}"


NEXT_STUBS = []                                      # (label, return label) of every switch to the next chunk


def dma_groups(stage):
    """The direct-to-LDS loads of one K / V tile into LDS stage `stage`: one [M0 setup, gap, load] group per load."""
    g = []
    for j in range(NDMA):
        g.append([f"s_add_u32 m0, {sr(T_M0)}, {KT(stage) + 4096 * j}", "s_nop 0",
                  f"global_load_lds_dwordx4 {vr(KOFF + j)}, {sr(D_KPTR, 2)}"])
        g.append([f"s_add_u32 m0, {sr(T_M0)}, {VT(stage) + 4096 * j}", "s_nop 0",
                  f"global_load_lds_dwordx4 {vr(VOFF + j)}, {sr(D_VPTR, 2)}"])
    return g


def advance_lines(e):
    """Move the K / V stream to the next tile of the walk (it stays on the last tile once all S_NT tiles have been
    requested).  The common path falls through; the switch to the next chunk of the table sits out of line."""
    l_skip, l_next = e.label("skip"), e.label("nextchunk")
    NEXT_STUBS.append((l_next, l_skip))
    return [f"s_add_u32 {sr(T_X)}, {sr(D_IDX)}, 1",
            f"s_cmp_ge_u32 {sr(T_X)}, {sr(S_NT)}",
            f"s_cbranch_scc1 {l_skip}",
            f"s_mov_b32 {sr(D_IDX)}, {sr(T_X)}",
            f"s_sub_u32 {sr(D_LEFT)}, {sr(D_LEFT)}, 1",
            f"s_cmp_eq_u32 {sr(D_LEFT)}, 0",
            f"s_cbranch_scc1 {l_next}",
            f"s_add_u32 {sr(D_KPTR)}, {sr(D_KPTR)}, {sr(S_KTILE)}",
            f"s_addc_u32 {sr(D_KPTR + 1)}, {sr(D_KPTR + 1)}, 0",
            f"s_add_u32 {sr(D_VPTR)}, {sr(D_VPTR)}, {sr(S_VTILE)}",
            f"s_addc_u32 {sr(D_VPTR + 1)}, {sr(D_VPTR + 1)}, 0",
            l_skip + ":"]


def gen_dma(e, stage):
    """Request a tile and advance the stream, in one piece (prologue)."""
    for grp in dma_groups(stage):
        for ln in grp:
            e.raw(ln)
    for ln in advance_lines(e):
        e.raw(ln)


def gen_table_entry(e):
    """Load the chunk-table entry at D_TBL into the DMA stream state (drains the LDS queue on this path)."""
    e.raw(f"v_mov_b32 {vr(TMP)}, {sr(D_TBL)}")
    e.raw(f"ds_read_b128 {vr(TMP + 2, 4)}, {vr(TMP)}")
    e.raw(f"ds_read_b32 {vr(TMP + 6)}, {vr(TMP)} offset:16")
    e.raw("s_waitcnt lgkmcnt(0)")
    for i, dst in enumerate((D_KPTR, D_KPTR + 1, D_VPTR, D_VPTR + 1, D_LEFT)):
        e.raw(f"v_readfirstlane_b32 {sr(dst)}, {vr(TMP + 2 + i)}")
    e.raw(f"s_add_u32 {sr(D_TBL)}, {sr(D_TBL)}, 32")


def generate():
    e = Emitter()
    p = Pipe(e)
    e.comment("---- prologue")
    e.raw(f"s_lshl_b32 {sr(T_M0)}, {sr(S_WAVE)}, 10")
    e.raw(f"s_add_u32 {sr(T_M0)}, {sr(T_M0)}, {sr(S_LDS)}")
    e.raw(f"s_mov_b32 {sr(T_REM)}, {sr(S_NT)}")
    e.raw(f"s_mov_b32 {sr(D_IDX)}, 0")
    e.raw(f"s_mov_b32 {sr(D_TBL)}, {sr(S_TBL)}")
    e.raw(f"v_mov_b32 {vr(TMP)}, 0x3fb8aa3b")
    e.raw(f"v_mul_f32 {vr(TMP)}, {sr(S_SCALE)}, {vr(TMP)}")
    e.raw("s_nop 0")
    e.raw(f"v_readfirstlane_b32 {sr(S_CEXP)}, {vr(TMP)}")
    e.comment("per-lane DMA offsets: instruction 4 j + wave covers rows 16 j + 4 wave .. + 3 of a 64-row tile")
    e.raw(f"v_mov_b32 {vr(KOFF)}, {vr(I_KOFF0)}")
    e.raw(f"v_mov_b32 {vr(VOFF)}, {vr(I_VOFF0)}")
    e.raw(f"v_mov_b32 {vr(DQOFF)}, {vr(I_DQOFF)}")
    for j in range(1, NDMA):
        e.raw(f"v_add_u32 {vr(KOFF + j)}, {sr(S_KRS16)}, {vr(KOFF + j - 1)}")
        e.raw(f"v_add_u32 {vr(VOFF + j)}, {sr(S_VRS16)}, {vr(VOFF + j - 1)}")
    gen_table_entry(e)
    for st in range(3):
        gen_dma(e, st)
    e.comment("Q / dO fragments (B operands) -> AGPRs; lane = query column, elements 16 ks + 8 (lane / 32) .. + 7")
    for qb, (qrow, dorow) in enumerate(((I_QROW0, I_DOROW0), (I_QROW1, I_DOROW1))):
        for ks in range(KS):
            e.raw(f"global_load_dwordx4 {vr(4 * (KS * qb + ks), 4)}, {vr(qrow, 2)}, off offset:{32 * ks}")
            e.raw(f"global_load_dwordx4 {vr(64 + 4 * (KS * qb + ks), 4)}, {vr(dorow, 2)}, off offset:{32 * ks}")
    e.comment("LDS offsets: x[ks] = xbase + (gf16 ^ 32 ks); transpose reads: trbase + (lf16 ^ 64 db), second half 8 rows down")
    for ks in range(KS):
        e.raw(f"v_xor_b32 {vr(TMP)}, {32 * ks}, {vr(I_GF16)}")
        e.raw(f"v_add_u32 {vr(XL + ks)}, {vr(I_XBASE)}, {vr(TMP)}")
        if SPLIT:
            e.raw(f"v_add_u32 {vr(XH + ks)}, 0x10000, {vr(XL + ks)}")
    for db in range(DB):
        e.raw(f"v_xor_b32 {vr(TMP)}, {64 * db}, {vr(I_LF16)}")
        e.raw(f"v_add_u32 {vr(TRLO_L + db)}, {vr(I_TRBASE)}, {vr(TMP)}")
        e.raw(f"v_xor_b32 {vr(TMP)}, {(64 * db) ^ 32}, {vr(I_LF16)}")
        e.raw(f"v_add_u32 {vr(TRHI_L + db)}, {vr(I_TRBASE)}, {vr(TMP)}")
        e.raw(f"v_add_u32 {vr(TRHI_L + db)}, {8 * ROW}, {vr(TRHI_L + db)}")
        if SPLIT:
            e.raw(f"v_add_u32 {vr(TRLO_H + db)}, 0x10000, {vr(TRLO_L + db)}")
            e.raw(f"v_add_u32 {vr(TRHI_H + db)}, 0x10000, {vr(TRHI_L + db)}")
    for i in range(32 * DB):
        e.raw(f"v_accvgpr_write_b32 {ar(i)}, 0")
    e.raw("s_waitcnt vmcnt(0)")
    e.comment("Q <- bf16(Q * scale * log2(e)): the S^T MFMAs then deliver exponents in log2 units")
    for i in range(0, 8 * KS, 4):
        for j in range(4):
            e.raw(f"v_lshlrev_b32 {vr(PT + 2 * j)}, 16, {vr(i + j)}")
            e.raw(f"v_and_b32 {vr(PT + 1 + 2 * j)}, 0xffff0000, {vr(i + j)}")
        for j in range(8):
            e.raw(f"v_mul_f32 {vr(PT + j)}, {sr(S_CEXP)}, {vr(PT + j)}")
        for j in range(4):
            e.raw(f"v_cvt_pk_bf16_f32 {vr(i + j)}, {vr(PT + 2 * j)}, {vr(PT + 1 + 2 * j)}")
    for i in range(8 * KS):
        e.raw(f"v_accvgpr_write_b32 {ar(128 + i)}, {vr(i)}")
        e.raw(f"v_accvgpr_write_b32 {ar(192 + i)}, {vr(64 + i)}")
    for qb, src in ((0, I_ND0), (1, I_ND1)):
        for v in range(16):
            e.raw(f"v_mov_b32 {vr(ND(qb) + v)}, {vr(src)}")
    for qb, src in ((0, I_NL0), (1, I_NL1)):
        for v in range(16):
            e.raw(f"v_mov_b32 {vr(NL(qb) + v)}, {vr(src)}")
    e.raw("s_barrier")
    e.comment("pipeline fill: S^T, P and dP' of block (0, 0)")
    gen_block(p, None, (0, 0), (0, 1), 1, 0, do_b=False, prefetched=False)

    l_loop, l_done = e.label("loop"), e.label("done")
    drains = []
    e.raw(l_loop + ":")
    loop_entry = list(e.ds)
    seq = 1
    for u in range(NS):
        un = (u + 1) % NS

        def head(u=u):
            # tile T + 1 has landed everywhere and nobody reads tile T - 1 any more: tile T + 3 may be requested
            e.raw(f"s_waitcnt vmcnt({2 * NDMA})")
            e.raw("s_barrier")
        side = {k: grp for k, grp in enumerate(dma_groups((u + 3) % NS))}
        side[2 * NDMA] = advance_lines(e)
        # the head sits between the tail prefetch of the block before and this block's first MFMA
        gen_block(p, (u, 0), (u, 1), (un, 0), 0, seq, head=head, side=side)
        seq += 1
        l_drain = e.label("drain")
        e.raw(f"s_cmp_eq_u32 {sr(T_REM)}, 1")
        e.raw(f"s_cbranch_scc1 {l_drain}")
        drains.append((l_drain, u, list(e.ds), dict(p.frag_reg), dict(p.uses_left), dict(p.owner), seq))
        gen_block(p, (u, 1), (un, 0), (un, 1), 1, seq)
        seq += 1
        e.raw(f"s_sub_u32 {sr(T_REM)}, {sr(T_REM)}, 1")
    assert [t.split("_", 1)[1] for t in e.ds] == [t.split("_", 1)[1] for t in loop_entry], (e.ds, loop_entry)
    e.raw(f"s_branch {l_loop}")
    for l_drain, u, ds, fr, ul, ow, sq in drains:
        e.raw(l_drain + ":")
        e.ds, p.frag_reg, p.uses_left, p.owner = list(ds), dict(fr), dict(ul), dict(ow)
        for t in p.uses_left:
            p.uses_left[t] = 0          # prefetched fragments of a block that does not exist
        e.raw("s_nop 7")                # dP' of the last block was written by the MFMAs just issued
        e.raw("s_nop 7")
        gen_block(p, (u, 1), None, None, 1, sq, do_ac=False)
        e.raw(f"s_branch {l_done}")
    for l_next, l_skip in NEXT_STUBS:
        e.raw(l_next + ":")
        gen_table_entry(e)
        e.raw(f"s_branch {l_skip}")
    e.raw(l_done + ":")
    e.raw("s_waitcnt vmcnt(0) lgkmcnt(0)")
    e.comment("---- epilogue: dq_acc += scale * dQ; lane = query row, 4 consecutive d per 16-byte access")
    e.raw("s_nop 7")
    e.raw("s_nop 7")
    for qb in range(QB):
        if qb == 1:
            e.raw(f"v_add_u32 {vr(DQOFF)}, {sr(S_DQQB)}, {vr(DQOFF)}")
        for db in range(DB):
            for j in range(4):
                e.raw(f"global_load_dwordx4 {vr(4 * (4 * db + j), 4)}, {vr(DQOFF)}, {sr(S_DQPTR, 2)} offset:{128 * db + 32 * j}")
        for db in range(DB):
            for j in range(4):
                t = 4 * (4 * db + j)
                e.raw(f"s_waitcnt vmcnt({4 * DB - 1 - (4 * db + j)})")
                for i in range(4):
                    e.raw(f"v_accvgpr_read_b32 {vr(TMP)}, {ar(ACC(db, qb) + 4 * j + i)}")
                    e.raw("s_nop 0")
                    e.raw(f"v_fma_f32 {vr(t + i)}, {vr(TMP)}, {sr(S_SCALE)}, {vr(t + i)}")
        for db in range(DB):
            for j in range(4):
                e.raw(f"global_store_dwordx4 {vr(DQOFF)}, {vr(4 * (4 * db + j), 4)}, {sr(S_DQPTR, 2)} offset:{128 * db + 32 * j}")
        e.raw("s_waitcnt vmcnt(0)")
    return e


def main():
    e = generate()
    clob = [f"v{i}" for i in range(256) if not 160 <= i < 180] + [f"a{i}" for i in range(256)]
    clob += [f"s{S_CEXP}"] + [f"s{i}" for i in range(64, 76)]
    write_inc(sys.stdout, "gen_bwd_dq_asm.py" + (" 64" if D == 64 else ""), "ST_DQ_FAST" + ("64" if D == 64 else ""), e,
              LDS_BYTES, clob)


if __name__ == "__main__":
    main()
