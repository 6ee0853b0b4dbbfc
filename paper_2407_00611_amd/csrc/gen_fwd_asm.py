#!/usr/bin/env python3
"""Generates the gfx950 assembly of the forward main loop (head_dim 128, or 64) as a C string literal.

    python gen_fwd_asm.py > st_fwd_asm.inc          (build.py does this before compiling)
    python gen_fwd_asm.py 64 > st_fwd64_asm.inc     (head_dim 64: half the contraction steps and half the
                                                     O^T row blocks per key block, tiles of 128-byte rows)

Body of ONE `asm volatile` statement in st_fwd_fast.hip.  A workgroup (4 wavefronts) owns 256 queries of
one head, 64 per wavefront as two 32-query blocks, and walks the 64-key tiles that every one of its rows
sees in full; it writes the partial (O, lse) of those tiles.  Everything else (masked tiles, ragged tails,
ragged query tiles) is done afterwards by the general kernel, which folds its own partial state into this
one with the log-sum-exp merge.

MFMA C layout "lane = query column": the exponent reference r (log2 units) and the row sum are one
register per lane and query block.  The Q fragments are multiplied by scale * log2(e) once (and rounded
to bf16 again), and every S^T accumulator starts from -r instead of zero, so the MFMAs deliver the
exponent S c - r directly and no VALU instruction is spent on it.  The reference is lazy: it only moves, by a whole number of log2 units,
when a block's maximum exceeds it by more than GAP, so the rescale factor is an exact power of two and the
common path never touches the accumulators.

Per 32-key block i and wavefront two groups of 16 MFMAs, software-pipelined two blocks deep:
    group B   O^T += V^T P^T(i)          A: V^T of block i by LDS transpose reads, B: packed P(i)
    group A   S^T(i+2) = K Q^T           A: K rows of block i+2 from LDS,          B: Q fragments (AGPRs)
    VALU      slots 3..9: row maximum of S(i+1), both halves, and the test against the reference
              (rare: call the rescale routine);  slots 10..31: P(i+1) = exp2(S c - r), bf16 pack, row sums
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
NSLOT = 4 * DB + 2 * KS                              # MFMAs per key block and wavefront
SPLIT = 4 * 2 * TILE > 65536                         # ring beyond the 16-bit offset field: second set of base registers
                                                     # (GAP, log2 units a block maximum may exceed the reference by, arrives in s46)

# ---- AGPRs
def ACC(db, qb): return 16 * (2 * db + qb)
def QF(qb, ks): return 128 + 4 * (KS * qb + ks)

# ---- VGPRs
def SBUF(buf, qb): return 32 * buf + 16 * qb        # two score buffers (S, then P in fp32)
def P16(buf, qb, m): return 64 + 16 * buf + 8 * qb + 4 * m
def NL(qb): return 240 - 16 * qb                     # sixteen copies of -r (minus the exponent reference, log2 units):
                                                     # the C operand that starts every S^T accumulator
                                                     # (NL(1) reuses the input registers once the prologue has read them)
def LSUM(qb, m, c=0): return (98 if c == 0 else 194) + 2 * qb + m   # partial row sums (this lane's key rows), two chains each
def MX(qb): return 102 + qb                         # block maximum, then d = max * c - r
GAPR, DMAX = 105, 106                                # GAP; max over both query blocks of d
TMP = 108                                            # 108..119
POOL0 = 120                                          # 2 rings x 4 fragments x 4 registers
XL, XH = 152, 160
TRLO_L, TRHI_L, TRLO_H, TRHI_H = 168, 172, 176, 180
KOFF, VOFF = 184, 188
OOFF, LSEOFF = 192, 193
RT = 200                                             # 200..223: temporaries of the rescale routine
# inputs (pinned by the C++ side): v[224:239]
I_QROW0, I_QROW1, I_XBASE, I_GF16, I_TRBASE, I_LF16, I_KOFF0, I_VOFF0, I_OOFF, I_LSEOFF = (
    224, 226, 228, 229, 230, 231, 232, 233, 234, 235)
S_GAP = 46
(S_LDS, S_WAVE, S_NT, S_KRS16, S_VRS16, S_SCALE, S_OPTR, S_OQB, S_TBL, S_KTILE, S_VTILE, S_LSEPTR) = (
    32, 33, 34, 35, 36, 37, 38, 40, 41, 42, 43, 44)
# scalar temporaries
S_CEXP, T_M0, T_REM, D_KPTR, D_VPTR, D_LEFT, D_IDX, D_TBL, T_X = 47, 64, 65, 66, 68, 70, 71, 72, 73
T_RET, T_RARE = 76, 78                               # return address; address of rescale routine b at 78 + 2 b

# ---- LDS map
def KT(s): return 2 * TILE * s
def VT(s): return 2 * TILE * s + TILE
TBL = 2 * TILE * NS
LDS_BYTES = TBL + 2048

LAT = int(os.environ.get("ST_GEN_FWD_LAT", 3))
BUDGET = int(os.environ.get("ST_GEN_FWD_BUDGET", 6 if D == 128 else 13))
BRANCH_SLOT = 2 * DB + 1                             # the reference test sits behind this MFMA slot (m = 1, db = 0 issued)


NEXT_STUBS = []                                      # (label, return label) of every switch to the next chunk
STUBS = []                                           # (call label, return label, P buffer) of every reference test


class Pipe:
    def __init__(self, e):
        self.e = e
        self.frag_reg, self.uses_left, self.owner = {}, {}, {}

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

    def snapshot(self):
        return list(self.e.ds), dict(self.frag_reg), dict(self.uses_left), dict(self.owner)

    def restore(self, snap):
        self.e.ds, self.frag_reg, self.uses_left, self.owner = list(snap[0]), dict(snap[1]), dict(snap[2]), dict(snap[3])


def upper(stage): return SPLIT and stage >= 2
def xreg(stage, ks): return (XH if upper(stage) else XL) + ks
def trregs(stage): return (TRLO_H, TRHI_H) if upper(stage) else (TRLO_L, TRHI_L)
def imm(stage, base): return base - (65536 if upper(stage) else 0)


def read_k(p, blk, ks, seq):
    stage, kb = blk
    tag = f"k{seq}_{ks}"
    r = p.alloc(0, ks, tag, QB)
    p.e.ds_read(f"ds_read_b128 {vr(r, 4)}, {vr(xreg(stage, ks))} offset:{imm(stage, KT(stage)) + 32 * ROW * kb}", tag)


def read_vt(p, blk, m, db, seq):
    """V^T fragment (32 d rows x 16 keys) of a block: A operand of O^T += V^T P^T."""
    stage, kb = blk
    tag = f"t{seq}_{m}_{db}"
    r = p.alloc(1, DB * m + db, tag, QB)
    lo, hi = trregs(stage)
    off = imm(stage, VT(stage)) + 32 * ROW * kb + 16 * ROW * m
    p.e.ds_read(f"ds_read_b64_tr_b16 {vr(r, 2)}, {vr(lo + db)} offset:{off}", tag + "lo")
    p.e.ds_read(f"ds_read_b64_tr_b16 {vr(r + 2, 2)}, {vr(hi + db)} offset:{off}", tag)


def valu_max(buf, full=False):
    """d = maximum of the exponents S c - r in buffer `buf` over this lane's key rows (full: over both halves of the
    wavefront, i.e. the whole block), per query block.  The test against GAP is a wavefront-wide vote, so the
    common path does not need the halves combined."""
    out = []
    for qb in range(QB):
        s0 = SBUF(buf, qb)
        out.append(f"v_max3_f32 {vr(MX(qb))}, {vr(s0)}, {vr(s0 + 1)}, {vr(s0 + 2)}")
        for v in range(3, 15, 2):
            out.append(f"v_max3_f32 {vr(MX(qb))}, {vr(MX(qb))}, {vr(s0 + v)}, {vr(s0 + v + 1)}")
        out.append(f"v_max_f32 {vr(MX(qb))}, {vr(MX(qb))}, {vr(s0 + 15)}")
    if full:
        out += valu_exchange()
    out.append(f"v_max_f32 {vr(DMAX)}, {vr(MX(0))}, {vr(MX(1))}")
    return out


def valu_exchange():
    """The two halves of the wavefront hold different key rows of the same query column: make MX the maximum of both."""
    out = []
    for qb in range(QB):
        out.append(f"v_mov_b32 {vr(TMP + qb)}, {vr(MX(qb))}")
    out.append("s_nop 1")
    for qb in range(QB):
        out.append(f"v_permlane32_swap_b32 {vr(TMP + qb)}, {vr(MX(qb))}")
    out.append("s_nop 1")
    for qb in range(QB):
        out.append(f"v_max_f32 {vr(MX(qb))}, {vr(MX(qb))}, {vr(TMP + qb)}")
    return out


def valu_exp(sbuf, pbuf):
    """P = exp2(exponent) in place, packed to bf16 into P buffer `pbuf`, row sums of the fp32 values (plain adds
    in two chains per group: measured cheaper than v_dot2c_f32_bf16 on the packed values against ones)."""
    out = []
    for qb in range(QB):
        for m in range(2):
            rs = [SBUF(sbuf, qb) + 8 * m + i for i in range(8)]
            for r in rs:
                out.append((f"v_exp_f32 {vr(r)}, {vr(r)}", (), 2))
            for i in range(4):
                d = P16(pbuf, qb, m) + i
                out.append((f"v_cvt_pk_bf16_f32 {vr(d)}, {vr(rs[2 * i])}, {vr(rs[2 * i + 1])}", (d,), 1))
            for i in range(8):
                out.append((f"v_add_f32 {vr(LSUM(qb, m, i % 2))}, {vr(LSUM(qb, m, i % 2))}, {vr(rs[i])}", (), 1))
    return out


def gen_iter(p, cur, nxt, nxt2, par, seq, do_a=True, do_valu=True, head=None, prefetch=True, side=None):
    """Block i = cur, i+1 = nxt (its V^T is prefetched at the tail), i+2 = nxt2 (its K feeds group A).
    par = i % 2: P(i) sits in P buffer par, S(i+1) in score buffer 1 - par, S(i+2) goes to score buffer par."""
    e = p.e
    e.comment(f"======== block {cur}: O^T += V^T P^T{cur} | S^T{nxt2} -> buffer {par} | softmax of {nxt}")
    reads = {k: [] for k in range(-1, NSLOT)}

    def plan(first_use, fn):
        reads[max(first_use - LAT, -1)].append(fn)

    slots = []
    for m in range(2):
        for db in range(DB):
            k = 2 * (DB * m + db)
            if not (m == 0 and db < 2):                   # requested at the tail of the block before
                plan(k, (lambda m=m, db=db: read_vt(p, cur, m, db, seq)))
            for qb in range(QB):
                slots.append(("B", m, db, qb))
    if do_a:
        for ks in range(KS):
            plan(4 * DB + 2 * ks, (lambda ks=ks: read_k(p, nxt2, ks, seq)))
            for qb in range(QB):
                slots.append(("A", ks, qb))
    else:
        slots += [None] * (2 * KS)
    if prefetch and nxt is not None:
        for db in range(2):
            reads[NSLOT - 3 + db].append(lambda db=db: read_vt(p, nxt, 0, db, seq + 1))

    valu_m = valu_max(1 - par) if do_valu else []
    valu_e = valu_exp(1 - par, 1 - par) if do_valu else []
    mi, vi = [0], [0]

    if head is not None:
        head()
    for fn in reads[-1]:
        fn()
    for k, sl in enumerate(slots):
        if sl is not None and sl[0] == "B":
            _, m, db, qb = sl
            tag = f"t{seq}_{m}_{db}"
            e.need(tag)
            acc = ar(ACC(db, qb), 16)
            e.mfma(acc, vr(p.use(tag), 4), vr(P16(par, qb, m), 4), acc)
        elif sl is not None:
            _, ks, qb = sl
            tag = f"k{seq}_{ks}"
            e.need(tag)
            d = vr(SBUF(par, qb), 16)
            e.mfma(d, vr(p.use(tag), 4), ar(QF(qb, ks), 4), vr(NL(qb), 16) if ks == 0 else d)
        units = 0
        for fn in reads[k]:
            n0 = len(e.ds)
            fn()
            units += len(e.ds) - n0
        if side and k in side:                           # tile request / stream bookkeeping spread under the MFMAs
            for ln in side[k]:
                e.raw(ln)
            units += 2
        if do_valu:
            # S(i+1) was written by the last group of the block before: first reader three MFMA issues later
            while 3 <= k <= BRANCH_SLOT and mi[0] < len(valu_m) and (units < BUDGET or k == BRANCH_SLOT):
                e.raw(valu_m[mi[0]])
                mi[0] += 1
                units += 1
            if k == BRANCH_SLOT:
                # the common path falls through; the call sits out of line behind the loop (a taken branch costs a refetch)
                l_call, l_back = e.label("call"), e.label("back")
                e.raw(f"v_cmp_gt_f32 vcc, {vr(DMAX)}, {vr(GAPR)}")
                e.raw("s_cmp_lg_u64 vcc, 0")
                e.raw(f"s_cbranch_scc1 {l_call}")
                e.raw(l_back + ":")
                STUBS.append((l_call, l_back, par))
            while k > BRANCH_SLOT and vi[0] < len(valu_e) and units + valu_e[vi[0]][2] <= BUDGET:
                e.valu(valu_e[vi[0]][0], valu_e[vi[0]][1])
                units += valu_e[vi[0]][2]
                vi[0] += 1
    leftover = len(valu_e) - vi[0]
    while vi[0] < len(valu_e):           # what did not fit under the MFMAs (the pipeline stalls on it)
        e.valu(valu_e[vi[0]][0], valu_e[vi[0]][1])
        vi[0] += 1
    return leftover if do_a else 0


def gen_rescale_routine(e, pbuf):
    """Called when some row's block maximum exceeds its reference by more than GAP.  MFMA slots 0..BRANCH_SLOT of
    the calling block have been issued (all of m = 0 and db = 0 of m = 1); the rest of m = 1 still reads P buffer
    `pbuf`; the exponents in score buffer 1 - pbuf wait for their softmax.  Moves the reference of the jumping rows
    up by k = ceil(d) log2 units: accumulators, row sums and the pending packed P values are multiplied by 2^-k
    (exact), k is taken off the waiting exponents and off the start values of the S^T accumulators."""
    e.raw("s_nop 7")
    e.raw("s_nop 7")
    e.raw("s_nop 7")
    for ln in valu_exchange():          # both halves of a query column must move their reference by the same amount
        e.raw(ln)
    alpha = [RT, RT + 1]
    for qb in range(QB):
        k, ki = RT + 2 + qb, RT + 4 + qb
        e.raw(f"v_ceil_f32 {vr(k)}, {vr(MX(qb))}")
        e.raw(f"v_cmp_gt_f32 vcc, {vr(MX(qb))}, {vr(GAPR)}")
        e.raw("s_nop 1")
        e.raw(f"v_cndmask_b32 {vr(k)}, 0, {vr(k)}, vcc")
        for v in range(16):
            e.raw(f"v_sub_f32 {vr(NL(qb) + v)}, {vr(NL(qb) + v)}, {vr(k)}")
        for v in range(16):             # exponents of the block whose softmax comes next: they carry the old reference
            e.raw(f"v_sub_f32 {vr(SBUF(1 - pbuf, qb) + v)}, {vr(SBUF(1 - pbuf, qb) + v)}, {vr(k)}")
        e.raw(f"v_cvt_i32_f32 {vr(ki)}, {vr(k)}")
        e.raw(f"v_sub_u32 {vr(ki)}, 0, {vr(ki)}")
        e.raw(f"v_ldexp_f32 {vr(alpha[qb])}, 1.0, {vr(ki)}")
        for m in range(2):
            for c in range(2):
                e.raw(f"v_mul_f32 {vr(LSUM(qb, m, c))}, {vr(alpha[qb])}, {vr(LSUM(qb, m, c))}")
    t = RT + 8
    for qb in range(QB):
        for db in range(DB):
            for v0 in range(0, 16, 8):
                for i in range(8):
                    e.raw(f"v_accvgpr_read_b32 {vr(t + i)}, {ar(ACC(db, qb) + v0 + i)}")
                for i in range(8):
                    e.raw(f"v_mul_f32 {vr(t + i)}, {vr(alpha[qb])}, {vr(t + i)}")
                for i in range(8):
                    e.raw(f"v_accvgpr_write_b32 {ar(ACC(db, qb) + v0 + i)}, {vr(t + i)}")
        for i in range(4):                                   # pending packed P values: m = 1
            pr = P16(pbuf, qb, 1) + i
            e.raw(f"v_lshlrev_b32 {vr(t)}, 16, {vr(pr)}")
            e.raw(f"v_and_b32 {vr(t + 1)}, 0xffff0000, {vr(pr)}")
            e.raw(f"v_mul_f32 {vr(t)}, {vr(alpha[qb])}, {vr(t)}")
            e.raw(f"v_mul_f32 {vr(t + 1)}, {vr(alpha[qb])}, {vr(t + 1)}")
            e.raw(f"v_cvt_pk_bf16_f32 {vr(pr)}, {vr(t)}, {vr(t + 1)}")
    e.raw("s_nop 3")
    e.raw(f"s_setpc_b64 {sr(T_RET, 2)}")


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
    l_rare = [e.label("rescale0"), e.label("rescale1")]
    e.comment("---- prologue")
    e.raw(f"s_lshl_b32 {sr(T_M0)}, {sr(S_WAVE)}, 10")
    e.raw(f"s_add_u32 {sr(T_M0)}, {sr(T_M0)}, {sr(S_LDS)}")
    e.raw(f"s_mov_b32 {sr(T_REM)}, {sr(S_NT)}")
    e.raw(f"s_mov_b32 {sr(D_IDX)}, 0")
    e.raw(f"s_mov_b32 {sr(D_TBL)}, {sr(S_TBL)}")
    for b in range(2):          # addresses of the two rescale routines
        l_here = e.label("here")
        e.raw(f"s_getpc_b64 {sr(T_RARE + 2 * b, 2)}")
        e.raw(l_here + ":")
        e.raw(f"s_add_u32 {sr(T_RARE + 2 * b)}, {sr(T_RARE + 2 * b)}, {l_rare[b]}-{l_here}")
        e.raw(f"s_addc_u32 {sr(T_RARE + 2 * b + 1)}, {sr(T_RARE + 2 * b + 1)}, 0")
    e.raw(f"v_mov_b32 {vr(TMP)}, 0x3fb8aa3b")
    e.raw(f"v_mul_f32 {vr(TMP)}, {sr(S_SCALE)}, {vr(TMP)}")
    e.raw("s_nop 0")
    e.raw(f"v_readfirstlane_b32 {sr(S_CEXP)}, {vr(TMP)}")
    e.raw(f"v_mov_b32 {vr(GAPR)}, {sr(S_GAP)}")
    e.raw(f"v_mov_b32 {vr(KOFF)}, {vr(I_KOFF0)}")
    e.raw(f"v_mov_b32 {vr(VOFF)}, {vr(I_VOFF0)}")
    e.raw(f"v_mov_b32 {vr(OOFF)}, {vr(I_OOFF)}")
    e.raw(f"v_mov_b32 {vr(LSEOFF)}, {vr(I_LSEOFF)}")
    for j in range(1, NDMA):
        e.raw(f"v_add_u32 {vr(KOFF + j)}, {sr(S_KRS16)}, {vr(KOFF + j - 1)}")
        e.raw(f"v_add_u32 {vr(VOFF + j)}, {sr(S_VRS16)}, {vr(VOFF + j - 1)}")
    gen_table_entry(e)
    for st in range(3):
        gen_dma(e, st)
    e.comment("Q fragments (B operands) -> AGPRs; lane = query column, elements 16 ks + 8 (lane / 32) .. + 7")
    for qb, qrow in enumerate((I_QROW0, I_QROW1)):
        for ks in range(KS):
            e.raw(f"global_load_dwordx4 {vr(4 * (KS * qb + ks), 4)}, {vr(qrow, 2)}, off offset:{32 * ks}")
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
    for qb in range(QB):
        for m in range(2):
            for c in range(2):
                e.raw(f"v_mov_b32 {vr(LSUM(qb, m, c))}, 0")
    e.raw("s_waitcnt vmcnt(0)")
    e.comment("Q <- bf16(Q * scale * log2(e)): the MFMAs then deliver exponents in log2 units")
    for i in range(0, 8 * KS, 4):
        for j in range(4):
            e.raw(f"v_lshlrev_b32 {vr(64 + 2 * j)}, 16, {vr(i + j)}")
            e.raw(f"v_and_b32 {vr(65 + 2 * j)}, 0xffff0000, {vr(i + j)}")
        for j in range(8):
            e.raw(f"v_mul_f32 {vr(64 + j)}, {sr(S_CEXP)}, {vr(64 + j)}")
        for j in range(4):
            e.raw(f"v_cvt_pk_bf16_f32 {vr(i + j)}, {vr(64 + 2 * j)}, {vr(65 + 2 * j)}")
    for i in range(8 * KS):
        e.raw(f"v_accvgpr_write_b32 {ar(128 + i)}, {vr(i)}")
    e.raw("s_barrier")

    e.comment("---- pipeline fill: exponents of block (0,0) from zero, reference, P and row sums; then block (0,1) from -r")

    def fill_s(blk, buf, seq, c_init):
        for ks in range(KS):
            read_k(p, blk, ks, seq)
            if ks % 4 == 3:
                for k2 in range(ks - 3, ks + 1):
                    e.need(f"k{seq}_{k2}")
                    for qb in range(QB):
                        d = vr(SBUF(buf, qb), 16)
                        e.mfma(d, vr(p.use(f"k{seq}_{k2}"), 4), ar(QF(qb, k2), 4), c_init(qb) if k2 == 0 else d)

    fill_s((0, 0), 0, -2, lambda qb: "0")
    e.raw("s_nop 7")
    e.raw("s_nop 7")
    for ln in valu_max(0, full=True):           # with r = 0: d = row maximum of S c
        e.raw(ln)
    for qb in range(QB):                        # reference = ceil(max), whole log2 units; shift block (0,0) by hand
        e.raw(f"v_ceil_f32 {vr(MX(qb))}, {vr(MX(qb))}")
        for v in range(16):
            e.raw(f"v_sub_f32 {vr(NL(qb) + v)}, 0, {vr(MX(qb))}")
        for v in range(16):
            e.raw(f"v_sub_f32 {vr(SBUF(0, qb) + v)}, {vr(SBUF(0, qb) + v)}, {vr(MX(qb))}")
    fill_s((0, 1), 1, -1, lambda qb: vr(NL(qb), 16))
    for text, writes, _ in valu_exp(0, 0):
        e.valu(text, writes)
    for db in range(2):
        read_vt(p, (0, 0), 0, db, 0)

    l_loop, l_done = e.label("loop"), e.label("done")
    e.raw(l_loop + ":")
    loop_entry = list(e.ds)
    drains = []
    seq = 0
    leftover = 0
    for u in range(NS):
        un = (u + 1) % NS
        l_drain = e.label("drain")
        e.raw(f"s_cmp_eq_u32 {sr(T_REM)}, 1")
        e.raw(f"s_cbranch_scc1 {l_drain}")
        drains.append((l_drain, u, p.snapshot(), seq))

        def head(u=u):
            # tile T + 1 has landed everywhere and nobody reads tile T - 1 any more: tile T + 3 may be requested
            e.raw(f"s_waitcnt vmcnt({2 * NDMA})")
            e.raw("s_barrier")
        side = {k: grp for k, grp in enumerate(dma_groups((u + 3) % NS))}
        side[2 * NDMA] = advance_lines(e)
        leftover += gen_iter(p, (u, 0), (u, 1), (un, 0), 0, seq, head=head, side=side)
        seq += 1
        leftover += gen_iter(p, (u, 1), (un, 0), (un, 1), 1, seq)
        seq += 1
        e.raw(f"s_sub_u32 {sr(T_REM)}, {sr(T_REM)}, 1")
    assert [t.split("_", 1)[1] for t in e.ds] == [t.split("_", 1)[1] for t in loop_entry], (e.ds, loop_entry)
    e.raw(f"s_branch {l_loop}")
    for l_drain, u, snap, sq in drains:
        e.raw(l_drain + ":")
        p.restore(snap)
        # the last tile: its second block still needs its softmax, nothing beyond it exists
        gen_iter(p, (u, 0), (u, 1), None, 0, sq, do_a=False)
        e.raw("s_nop 7")                 # the exponentials above were not hidden under a second MFMA group
        gen_iter(p, (u, 1), None, None, 1, sq + 1, do_a=False, do_valu=False, prefetch=False)
        e.raw(f"s_branch {l_done}")
    for l_next, l_skip in NEXT_STUBS:
        e.raw(l_next + ":")
        gen_table_entry(e)
        e.raw(f"s_branch {l_skip}")
    for l_call, l_back, par in STUBS:
        e.raw(l_call + ":")
        e.raw(f"s_swappc_b64 {sr(T_RET, 2)}, {sr(T_RARE + 2 * par, 2)}")
        e.raw(f"s_branch {l_back}")
    for b in range(2):
        e.raw(l_rare[b] + ":")
        gen_rescale_routine(e, b)
    e.raw(l_done + ":")
    e.raw("s_waitcnt vmcnt(0) lgkmcnt(0)")

    e.comment("---- epilogue: O = acc / l, lse = (log2(l) + r) ln 2; lane = query row, 4 consecutive d per 16-byte store")
    e.raw("s_nop 7")
    e.raw("s_nop 7")
    for qb in range(QB):
        l, t = TMP, TMP + 1
        e.raw(f"v_add_f32 {vr(l)}, {vr(LSUM(qb, 0))}, {vr(LSUM(qb, 1))}")
        e.raw(f"v_add_f32 {vr(t)}, {vr(LSUM(qb, 0, 1))}, {vr(LSUM(qb, 1, 1))}")
        e.raw(f"v_add_f32 {vr(l)}, {vr(l)}, {vr(t)}")
        e.raw(f"v_mov_b32 {vr(t)}, {vr(l)}")
        e.raw("s_nop 1")
        e.raw(f"v_permlane32_swap_b32 {vr(t)}, {vr(l)}")
        e.raw("s_nop 1")
        e.raw(f"v_add_f32 {vr(l)}, {vr(l)}, {vr(t)}")
        e.raw(f"v_rcp_f32 {vr(TMP + 2)}, {vr(l)}")
        e.raw(f"v_log_f32 {vr(TMP + 3)}, {vr(l)}")
        e.raw("s_nop 1")
        e.raw(f"v_sub_f32 {vr(TMP + 3)}, {vr(TMP + 3)}, {vr(NL(qb))}")
        e.raw(f"v_mul_f32 {vr(TMP + 3)}, 0x3f317218, {vr(TMP + 3)}")
        if qb == 1:
            e.raw(f"v_add_u32 {vr(OOFF)}, {sr(S_OQB)}, {vr(OOFF)}")
            e.raw(f"v_add_u32 {vr(LSEOFF)}, 128, {vr(LSEOFF)}")
        for db in range(DB):
            for j in range(4):
                t0 = 4 * (4 * db + j)
                for i in range(4):
                    e.raw(f"v_accvgpr_read_b32 {vr(t0 + i)}, {ar(ACC(db, qb) + 4 * j + i)}")
                e.raw("s_nop 0")
                for i in range(4):
                    e.raw(f"v_mul_f32 {vr(t0 + i)}, {vr(TMP + 2)}, {vr(t0 + i)}")
                e.raw(f"global_store_dwordx4 {vr(OOFF)}, {vr(t0, 4)}, {sr(S_OPTR, 2)} offset:{128 * db + 32 * j}")
        # lse: one lane per row (the lower half of the wavefront)
        e.raw(f"s_mov_b64 exec, 0xffffffff")
        e.raw(f"global_store_dword {vr(LSEOFF)}, {vr(TMP + 3)}, {sr(S_LSEPTR, 2)}")
        e.raw(f"s_mov_b64 exec, -1")
        e.raw("s_waitcnt vmcnt(0)")
    return e, leftover


def main():
    e, leftover = generate()
    if leftover:
        sys.stderr.write(f"gen_fwd_asm: {leftover} VALU instructions did not fit under the MFMAs\n")
    clob = [f"v{i}" for i in range(256) if not 224 <= i < 240] + [f"a{i}" for i in range(256)]
    clob += [f"s{S_CEXP}"] + [f"s{i}" for i in range(64, 82)]
    write_inc(sys.stdout, "gen_fwd_asm.py" + (" 64" if D == 64 else ""), "ST_FWD_FAST" + ("64" if D == 64 else ""), e,
              LDS_BYTES, clob)


if __name__ == "__main__":
    main()
