#!/usr/bin/env python3
"""Generates the gfx950 assembly of the dK/dV main loop (head_dim 128, or 64) as a C string literal.

    python gen_bwd_dkv_asm.py > st_bwd_dkv_asm.inc          (build.py does this before compiling)
    python gen_bwd_dkv_asm.py 64 > st_bwd_dkv64_asm.inc     (head_dim 64: half the MFMAs per phase, 128-byte tile rows)

The text is the body of ONE `asm volatile` statement in st_bwd_dkv_fast.hip.  The C++ kernel around it
computes addresses and hands them over in pinned registers (see IN_V / IN_S below); everything between
the K-fragment loads and the final read-modify-write of dK / dV is written here with hand-assigned
registers, because the kernel needs all 512 registers of a wavefront (256 accumulators in AGPRs, the
resident K fragments and the score tiles in VGPRs) and a fixed interleave of MFMA, LDS and VALU work.

Work of one workgroup (4 wavefronts): 256 keys of one KV head of one chunk (64 per wavefront), against a
run of 32-query blocks that see every one of those keys (no masking in here; blocks that need a mask go
to the general kernel).  Per block and wavefront, with the MFMA C layout "lane = key column":
    phase 1   E   = Q' K^T - lse log2e          A: Q' rows from LDS (Q' = bf16(Q scale log2 e), made once per backward
                                                by a pass of its own and shared with the other bf16 kernels, so that
                                                every kernel evaluates the same scores), B: resident K fragments,
                                                C init: -lse log2e
    phase 2   dP' = dO V^T - Delta              A: dO rows from LDS,       B: V rows from LDS, C init: -Delta
              VALU: P = exp2(E), bf16 pack                            (runs under phase 2 / 3 MFMAs)
    phase 3   dV^T += dO^T P                    A: dO^T by LDS transpose reads, B: packed P
              VALU: dS = P dP', bf16 pack (in place)                   (runs under phase 3 / 4 MFMAs)
    phase 4   dK^T += Q'^T dS                   A: Q'^T by LDS transpose reads, B: packed dS  (the epilogue's factor is
                                                ln 2 = scale / (scale log2 e) where dK = scale dS^T Q asks for scale)
The (head, block) pairs of a key tile are walked block by block from the LAST block down, the query heads of
the KV group being the inner index: workgroups of one XCD that work on key tiles of the same KV head then read
the same rows of Q' and dO at about the same time whichever block their own tile's run starts at (under a causal
mask the runs start at different blocks and all end at the last one), so those rows are fetched into the XCD's
L2 once per round of tiles instead of once per workgroup.
Q' / dO tiles arrive by direct global->LDS loads into a 4-stage ring, three blocks ahead; the per-row
statistics (lse, Delta) are loaded three blocks ahead into registers, transformed once and written to LDS
by every wavefront (identical values), so that no per-element VALU work is spent on them.

One barrier per block, in the middle of it (between phase 2 and phase 3): it publishes the next block's
tile and statistics and frees the stage of the block before, so the first LDS reads of the next block
are issued at the tail of this one and the MFMA stream runs across block boundaries.  The bookkeeping
of the four global pointers is branch-free scalar code spread under the MFMAs of phase 4.
"""
import os
import sys

from st_asmgen import Emitter, ar, sr, vr, write_inc

# ------------------------------------------------------------------------------------------------
# register map
# ------------------------------------------------------------------------------------------------
D = 64 if "64" in sys.argv[1:] else 128    # head_dim
NKB = 2          # 32-key blocks per wavefront
KS = D // 16     # contraction steps over head_dim (16 each)
DB = D // 32     # 32-row blocks of head_dim
NS = 4           # LDS stages of the Q / dO ring
PF = 3           # tiles in flight ahead of the one being computed
ROW = 2 * D      # bytes of one tile row in LDS
TQ = 32 * ROW    # one 32-query Q (or dO) tile
NDQ = TQ // 4096 # direct-to-LDS loads per wavefront and tile (4 wavefronts x 1 KiB each)
NREQ = 2 + 2 * NDQ                                   # memory operations of one block's request
P1, P2, P3, P4 = 0, 2 * KS, 4 * KS, 4 * KS + 4 * DB  # first MFMA slot of the four phases
NSLOT = 4 * KS + 8 * DB                              # MFMAs per block and wavefront

def KF(nb, ks): return 4 * (KS * nb + ks)            # v[KF : KF+3]
S0 = 64                                              # S[nb][v]  = v[64 + 16 nb + v]   (later P, fp32)
DP0 = 96                                             # dP[nb][v] = v[96 + 16 nb + v]   (later dS, then packed dS)
P16 = 128                                            # P16[nb][m] = v[128 + 8 nb + 4 m : +3]
ND = 128                                             # nd[v] = -Delta(row v): shares registers with P16 (dead from slot 18 on,
                                                     # P16 is first written later and last read in phase 3; nd is re-read at the tail)
NL = 144                                             # nl[v] = -lse(row v) * log2e
POOL0, NPOOL = 160, 12                               # fragment pool, 4 registers each; 48 fragments per block
ST = 208                                             # ST + 2 set + {0: lse, 1: Delta}
TMP = 212                                            # 212..214 temporaries, 215 = -inf
NINF = 215
X = 224                                              # x[ks]: natural-read offset inside a Q / dO tile
XV = 232                                             # xv[ks]: the same inside this wavefront's V rows
TRLO, TRHI = 240, 244                                # transpose-read offsets per d block
QOFF, DOOFF = 248, 250                               # per-lane global offsets of the two DMA instructions
STAT_G, STAT_L, DKV_OFF, G16 = 252, 253, 254, 255

# inputs pinned by the C++ side
IN_V = 176                                           # v[176:191]
(I_KROW0, I_KROW1, I_VOFF, I_QOFF0, I_QOFF1, I_DOOFF0, I_DOOFF1, I_STAT_G, I_DKV, I_XBASE, I_GF16, I_TRBASE,
 I_LF16, I_STAT_L) = (176, 178, 180, 181, 182, 183, 184, 185, 186, 187, 188, 189, 190, 191)
IN_SA, IN_SB = 32, 48                                # s[32:47], s[48:63]
S_QPTR, S_DOPTR, S_LSEPTR, S_DLPTR = 32, 34, 36, 38
# The walk over the (query head, 32-row block) pairs of a key tile has the head as its inner index: S_NIN heads
# per block, S_*IN bytes from one head to the next, S_*OUT bytes (signed, all three of one sign) from one block
# to the next one visited.
S_QIN, S_QOUT, S_DOIN, S_DOOUT, S_STOUT, S_NIN, S_NSTEPS, S_STIN = 40, 41, 42, 43, 44, 45, 46, 47
S_VPTR, S_VRS16, S_LDS, S_DKPTR, S_DVPTR, S_WAVE, S_RS32, S_SCALE = 48, 50, 51, 52, 54, 56, 57, 58
S_FLAGS, S_DKLP, S_DVLP = 59, 60, 62                # epilogue variant; bf16 copies of the dK / dV tile (if asked for)
# scalar temporaries (clobbered)
T_QPTR, T_QHEAD, T_DOPTR, T_DOHEAD = 64, 66, 68, 70
T_LSEPTR, T_LSEHEAD, T_DLPTR, T_DLHEAD = 72, 74, 76, 78
T_DBLK, T_DSTEP, T_ADV, T_WRAP, T_REM, T_M0, T_HIMASK, T_X, T_VPTR, T_INC, T_HINC = 80, 81, 82, 83, 84, 85, 86, 88, 90, 92, 93
T_HI, T_OHI = 94, 95                                 # upper half of the outer increment: this step's, and when one is applied

def ACC_K(db, nb): return 16 * (2 * db + nb)
def ACC_V(db, nb): return 128 + 16 * (2 * db + nb)

# LDS map (bytes, relative to the kernel's LDS base)
STATS = 0                                            # stage s: nl[32] at 256 s, nd[32] at 256 s + 128
def QT(s): return 1024 + 2 * TQ * s
def DOT(s): return 1024 + 2 * TQ * s + TQ
VT = 1024 + 2 * TQ * NS                              # V tile of the workgroup: 256 rows
LDS_BYTES = max(VT + 256 * ROW, 4 * 2 * 32 * (4 * D + 16))   # the tiles of the loop; the epilogue's staging rows

LAT = int(os.environ.get("ST_GEN_DKV_LAT", 3))          # MFMA slots between the issue of an LDS read and its first use
BUDGET = int(os.environ.get("ST_GEN_DKV_BUDGET", 6 if D == 128 else 11))       # issue units of side work per MFMA slot (an MFMA occupies the pipe for 8 quad-cycles)



STREAMS = ((T_QPTR, T_QHEAD, S_QIN, S_QOUT), (T_DOPTR, T_DOHEAD, S_DOIN, S_DOOUT),
           (T_LSEPTR, T_LSEHEAD, S_STIN, S_STOUT), (T_DLPTR, T_DLHEAD, S_STIN, S_STOUT))


def advance_code():
    """Branch-free move of the four global streams (Q', dO, lse, Delta) to the next (head, block) pair; they stay
    on the last one once all of them have been requested.  The inner increment (next head) is unsigned, the outer
    one (next block, applied to the base of the current block when the heads wrap) is a signed 32-bit number whose
    upper half T_OHI the prologue derives.  Only these instructions (and the loop control behind them) touch SCC
    between them, so they may be spread among non-scalar instructions."""
    c = [f"s_add_u32 {sr(T_X)}, {sr(T_DSTEP)}, 1",
         f"s_cmp_lt_u32 {sr(T_X)}, {sr(S_NSTEPS)}",
         f"s_cselect_b32 {sr(T_DSTEP)}, {sr(T_X)}, {sr(T_DSTEP)}",
         f"s_cselect_b32 {sr(T_ADV)}, 1, 0",
         f"s_add_u32 {sr(T_X)}, {sr(T_DBLK)}, {sr(T_ADV)}",
         f"s_cmp_eq_u32 {sr(T_X)}, {sr(S_NIN)}",                        # only possible when advancing
         f"s_cselect_b32 {sr(T_DBLK)}, 0, {sr(T_X)}",
         f"s_cselect_b32 {sr(T_WRAP)}, -1, 0",
         f"s_and_b32 {sr(T_HI)}, {sr(T_WRAP)}, {sr(T_OHI)}"]
    for ptr, head, bs, hs in STREAMS:
        c.append(f"s_mul_i32 {sr(T_INC)}, {sr(T_ADV)}, {sr(bs)}")
        c.append(f"s_and_b32 {sr(T_HINC)}, {sr(T_WRAP)}, {sr(hs)}")
        c += [f"s_add_u32 {sr(ptr)}, {sr(ptr)}, {sr(T_INC)}", f"s_addc_u32 {sr(ptr + 1)}, {sr(ptr + 1)}, 0",
              f"s_add_u32 {sr(head)}, {sr(head)}, {sr(T_HINC)}", f"s_addc_u32 {sr(head + 1)}, {sr(head + 1)}, {sr(T_HI)}"]
    c.append(f"s_cmp_lg_u32 {sr(T_WRAP)}, 0")
    for ptr, head, bs, hs in STREAMS:
        c.append(f"s_cselect_b64 {sr(ptr, 2)}, {sr(head, 2)}, {sr(ptr, 2)}")
    return c


def request_code(stage, st_set):
    """Statistics of a block into register set st_set, its Q / dO tile into LDS stage `stage` (6 memory operations)."""
    c = [[f"global_load_dword {vr(ST + 2 * st_set)}, {vr(STAT_G)}, {sr(T_LSEPTR, 2)}",
          f"global_load_dword {vr(ST + 2 * st_set + 1)}, {vr(STAT_G)}, {sr(T_DLPTR, 2)}"]]
    for ptr, off, tbase in ((T_QPTR, QOFF, QT(stage)), (T_DOPTR, DOOFF, DOT(stage))):
        for j in range(NDQ):
            c.append([f"s_add_u32 m0, {sr(T_M0)}, {tbase + 4096 * j}", "s_nop 0",
                      f"global_load_lds_dwordx4 {vr(off + j)}, {sr(ptr, 2)}"])
    return c


def stat_publish(e, st_set, stage, tag):
    """-lse log2(e) (or -inf for an empty row, whose P must be 0) and -Delta of the 32 rows to the stage's statistics slot."""
    rs = ST + 2 * st_set
    e.raw(f"v_mul_f32 {vr(TMP)}, 0xbfb8aa3b, {vr(rs)}")
    e.raw(f"v_xor_b32 {vr(TMP + 1)}, 0x80000000, {vr(rs + 1)}")
    e.raw(f"v_cmp_eq_f32 vcc, 0x7f800000, {vr(TMP)}")
    e.raw("s_nop 1")
    e.raw(f"v_cndmask_b32 {vr(TMP)}, {vr(TMP)}, {vr(NINF)}, vcc")
    e.raw(f"v_cndmask_b32_e64 {vr(TMP)}, {vr(TMP)}, {vr(TMP + 1)}, {sr(T_HIMASK, 2)}")
    e.ds_read(f"ds_write_b32 {vr(STAT_L)}, {vr(TMP)} offset:{STATS + 256 * stage}", tag)


class Pool:
    """Round-robin fragment registers; NPOOL divides the 48 fragments of a block, so every block sees the same map."""

    def __init__(self):
        self.next, self.owner, self.uses_left, self.reg = 0, {}, {}, {}

    def alloc(self, tag, uses):
        i = self.next % NPOOL
        self.next += 1
        old = self.owner.get(i)
        assert old is None or self.uses_left[old] == 0, f"fragment {old} overwritten by {tag} before its last use"
        self.owner[i], self.uses_left[tag], self.reg[tag] = tag, uses, POOL0 + 4 * i
        return POOL0 + 4 * i

    def use(self, tag):
        assert self.uses_left[tag] > 0, tag
        self.uses_left[tag] -= 1
        return self.reg[tag]


def plan_reads(e, pool, u, seq):
    """LDS reads of the block on stage u, by the MFMA slot behind which they are issued; negative slots are
    issued by the block before (slot + 64) or by the prologue."""
    qt, dot_, stats = QT(u), DOT(u), STATS + 256 * u
    reads = {k: [] for k in range(-EARLY, NSLOT)}

    def plan(first_use, fn):
        reads[first_use - LAT].append(fn)

    def rd_nat(tag, tile_imm, ks, xbase, uses):
        def f():
            r = pool.alloc(tag, uses)
            e.ds_read(f"ds_read_b128 {vr(r, 4)}, {vr(xbase + ks)} offset:{tile_imm}", tag)
        return f

    def rd_tr(tag, tile_imm, m, db):
        def f():
            r = pool.alloc(tag, NKB)
            e.ds_read(f"ds_read_b64_tr_b16 {vr(r, 2)}, {vr(TRLO + db)} offset:{tile_imm + 16 * ROW * m}", tag + "lo")
            e.ds_read(f"ds_read_b64_tr_b16 {vr(r + 2, 2)}, {vr(TRHI + db)} offset:{tile_imm + 16 * ROW * m}", tag)
        return f

    def rd_stat(tag, base_reg, imm, js):
        def f():
            for j in js:
                e.ds_read(f"ds_read_b128 {vr(base_reg + 4 * j, 4)}, {vr(G16)} offset:{imm + 32 * j}", f"{tag}{j}")
        return f

    for ks in range(KS):
        plan(2 * ks, rd_nat(f"{seq}q{ks}", qt, ks, X, NKB))
        if ks == 0:
            # the statistics were published before the barrier of the block before: read them early, two reads per
            # slot, instead of in one burst in front of the block (nl is free from slot 2 on, nd shares its registers
            # with the packed P, last read in phase 3)
            reads[-EARLY].append(rd_stat(f"{seq}nl", NL, stats, (0, 1)))
            reads[-EARLY + 1].append(rd_stat(f"{seq}nl", NL, stats, (2, 3)))
            reads[-EARLY + 4].append(rd_stat(f"{seq}nd", ND, stats + 128, (0, 1)))
            reads[-EARLY + 5].append(rd_stat(f"{seq}nd", ND, stats + 128, (2, 3)))
    for ks in range(KS):
        base = P2 + 2 * ks
        plan(base, rd_nat(f"{seq}do{ks}", dot_, ks, X, NKB))
        for nb in range(NKB):
            plan(base + nb, rd_nat(f"{seq}v{nb}_{ks}", 32 * ROW * nb, ks, XV, 1))
    for ph, tile in (("dV", dot_), ("dK", qt)):
        for m in range(2):
            for db in range(DB):
                base = (P3 if ph == "dV" else P4) + 2 * (DB * m + db)
                plan(base, rd_tr(f"{seq}{ph}t{m}_{db}", tile, m, db))
    return reads


EARLY = 12                # the next block's statistics are read from this many slots before the end of a block on
assert NSLOT - EARLY > P3 - 1 and NSLOT - EARLY + 4 >= P4, "statistics reads: behind the barrier, nd behind phase 3"
SYNC_SLOT = P3 - 1        # the barrier sits behind this MFMA slot (end of phase 2)
PUBLISH_SLOT = P3 - 6     # wait for the next block's loads and write its statistics behind this slot


def gen_step(e, pool, u, seq, reads, next_reads):
    """One 32-query block on LDS stage u (the loop is unrolled NS times so that stage addresses are immediates)."""
    e.comment(f"================ block on stage {u}")
    slots = []
    for ks in range(KS):
        for nb in range(NKB):
            slots.append(("S", ks, nb))
    for ks in range(KS):
        for nb in range(NKB):
            slots.append(("dP", ks, nb))
    for ph in ("dV", "dK"):
        for m in range(2):
            for db in range(DB):
                for nb in range(NKB):
                    slots.append((ph, m, db, nb))

    # ---- VALU work: (earliest slot, text, registers written, issue units, LDS tag it waits for)
    valu = []
    def S(nb, v): return S0 + 16 * nb + v
    def DP(nb, v): return DP0 + 16 * nb + v
    # VALU-1: P = exp2(E); pack P.  S[nb] is written by slot P2 - 2 + nb; its first reader comes three MFMA issues later.
    for m in range(2):
        for nb in range(NKB):
            early = P2 + 1 + nb
            for grp in range(2):
                vs = [8 * m + 4 * grp + i for i in range(4)]
                for v in vs:
                    valu.append((early, f"v_exp_f32 {vr(S(nb, v))}, {vr(S(nb, v))}", (), 2, None))
                if grp == 1:
                    for i in range(4):
                        d = P16 + 8 * nb + 4 * m + i
                        a = S(nb, 8 * m + 2 * i)
                        valu.append((max(early, P2 + 4), f"v_cvt_pk_bf16_f32 {vr(d)}, {vr(a)}, {vr(a + 1)}", (d,), 1, None))
    # VALU-2: dS = P dP', packed in place.  dP[nb] is written by slot P3 - 2 + nb; same distance.
    for m in range(2):
        for nb in range(NKB):
            early = P3 + 1 + nb
            for v in range(8 * m, 8 * m + 8):
                valu.append((early, f"v_mul_f32 {vr(DP(nb, v))}, {vr(S(nb, v))}, {vr(DP(nb, v))}", (), 1, None))
            for i in range(4):
                d = DP(nb, 4 * m + i)
                a = DP(nb, 8 * m + 2 * i)
                valu.append((early, f"v_cvt_pk_bf16_f32 {vr(d)}, {vr(a)}, {vr(a + 1)}", (d,), 1, None))
    vi = [0]
    produced = {}
    cur_slot = [0]

    def emit_valu(item):
        _, text, writes, units, needtag = item
        if needtag:
            assert False, "no VALU instruction reads the statistics any more"
            e.need(needtag)
        e.valu(text, writes)
        for r in writes:
            produced[r] = True
        return units

    def flush_until(regs):
        while not all(produced.get(r) for r in regs):
            assert vi[0] < len(valu), "packed operand never produced"
            emit_valu(valu[vi[0]])
            vi[0] += 1

    # scalar / memory side work behind fixed slots
    side = {k: [] for k in range(NSLOT)}
    req = request_code((u + PF) % NS, (u + 1) % 2)
    for i, grp in enumerate(req):                       # behind the barrier, one memory operation group per slot
        side[SYNC_SLOT + 1 + i] += grp
    adv = advance_code()
    per = 4 if D == 128 else 8
    for i in range(0, len(adv), per):                   # under phase 4, where the VALU is idle
        side[P4 + i // per] += adv[i:i + per]
    assert P4 + (len(adv) - 1) // per < NSLOT - 3

    stw = f"{seq}stw"
    for k, sl in enumerate(slots):
        ph = sl[0]
        cur_slot[0] = k
        if ph == "S":
            _, ks, nb = sl
            tag = f"{seq}q{ks}"
            e.need(tag)
            if ks == 0:
                e.need(f"{seq}nl3")
                c = vr(NL, 16)
            else:
                c = vr(S0 + 16 * nb, 16)
            e.mfma(vr(S0 + 16 * nb, 16), vr(pool.use(tag), 4), vr(KF(nb, ks), 4), c)
        elif ph == "dP":
            _, ks, nb = sl
            e.need(f"{seq}do{ks}")
            e.need(f"{seq}v{nb}_{ks}")
            if ks == 0:
                e.need(f"{seq}nd3")
                c = vr(ND, 16)
            else:
                c = vr(DP0 + 16 * nb, 16)
            a_reg = pool.use(f"{seq}do{ks}")
            e.mfma(vr(DP0 + 16 * nb, 16), vr(a_reg, 4), vr(pool.use(f"{seq}v{nb}_{ks}"), 4), c)
        else:
            _, m, db, nb = sl
            tag = f"{seq}{ph}t{m}_{db}"
            e.need(tag)
            if ph == "dV":
                b0, acc = P16 + 8 * nb + 4 * m, ACC_V(db, nb)
            else:
                b0, acc = DP0 + 16 * nb + 4 * m, ACC_K(db, nb)
            flush_until([b0 + i for i in range(4)])
            e.mfma(ar(acc, 16), vr(pool.use(tag), 4), vr(b0, 4), ar(acc, 16), breads=[b0 + i for i in range(4)])
        # ---- side work of this slot
        units = 0
        for fn in reads[k] + (next_reads[k - NSLOT] if k - NSLOT in next_reads else []):
            n0 = len(e.ds)
            fn()
            units += len(e.ds) - n0
        for ln in side[k]:
            e.raw(ln)
            units += 1
        if k == PUBLISH_SLOT:
            # tile and statistics of the next block: everything but the six newest memory operations has landed
            e.raw(f"s_waitcnt vmcnt({NREQ})")
            stat_publish(e, (u + 1) % 2, (u + 1) % NS, stw)
            units += 8
        while vi[0] < len(valu) and valu[vi[0]][0] <= k and units + valu[vi[0]][3] <= BUDGET:
            units += emit_valu(valu[vi[0]])
            vi[0] += 1
        if k == SYNC_SLOT:
            e.need(stw)
            e.raw("s_barrier")
    assert vi[0] == len(valu), f"VALU work left over: {len(valu) - vi[0]}"


class InFlight:
    """Memory operations of one counter in issue order (they complete in that order): need(tag) emits the wait
    that makes the tagged operation, and every older one, complete."""
    def __init__(self, e, counter, limit):
        self.e, self.counter, self.limit, self.q = e, counter, limit, []

    def issue(self, text, tag):
        if len(self.q) >= self.limit:                    # keep the hardware counter from saturating
            self.q = self.q[len(self.q) - self.limit // 2:]
            self.e.raw(f"s_waitcnt {self.counter}({len(self.q)})")
        self.e.raw(text)
        self.q.append(tag)

    def need(self, tag):
        if tag in self.q:
            self.q = self.q[self.q.index(tag) + 1:]
            assert len(self.q) <= (63 if self.counter == "vmcnt" else 15)
            self.e.raw(f"s_waitcnt {self.counter}({len(self.q)})")


def epilogue(e):
    """dk_acc (+)= scale * dK, dv_acc (+)= dV.  The accumulators hold dK^T / dV^T with lane = key, so a lane owns
    16-byte pieces of 32 different rows of the output: written like that, every access of a wavefront touches
    32 cache lines and the epilogue is bound by the rate of cache-line lookups.  Each wavefront therefore turns
    its tile through LDS (its own region, rows padded by 16 bytes) and reads, adds and writes the fp32
    accumulators in HBM as whole rows: 64 lanes x 16 bytes = RPI complete rows per access.
    Four passes (key block x {dK, dV}).  Four variants, chosen by S_FLAGS: bit 0 = the accumulators are assigned,
    not added to (nothing is read from HBM); bit 1 = the final values are also written rounded to bf16.  When
    adding, the HBM reads run two passes ahead of their use; nothing waits for the stores (vmcnt counts loads
    and stores in issue order, which is why every variant has its own waits)."""
    RSL = 4 * D + 16                                   # bytes of a padded fp32 row in LDS
    LPR = D // 4                                       # lanes per row
    RPI = 64 // LPR                                    # rows per access
    NLD = 32 // RPI                                    # accesses per pass
    LG = LPR.bit_length() - 1
    def G(p, n): return 4 * NLD * (p % 2) + 4 * n      # HBM values of pass p (two sets)
    def T(n): return 128 + 4 * n                       # the wavefront's own values, row layout
    def W(k): return 192 + 4 * (k % 4)                 # accumulator pieces on their way to LDS; later bf16 pairs
    LR, LW, GOFF, LANE, TA, TB, GOFF2 = 208, 209, 210, 211, 212, 213, 214
    PTL, PTS, STEP, SW, PTB, STEP2 = 64, 66, 68, 69, 70, 72   # scalar temporaries of the loop, free now
    e.comment("---- epilogue: dk_acc (+)= scale * dK, dv_acc (+)= dV, through LDS so that HBM sees whole rows")
    e.raw("s_nop 7")
    e.raw("s_nop 7")
    e.raw("s_barrier")                                 # every wavefront is done with the tiles in LDS
    e.raw(f"v_mbcnt_lo_u32_b32 {vr(LANE)}, -1, 0")
    e.raw(f"v_mbcnt_hi_u32_b32 {vr(LANE)}, -1, {vr(LANE)}")
    e.raw(f"s_lshr_b32 {sr(STEP)}, {sr(S_RS32)}, 5")                     # bytes of one output row
    e.raw(f"s_lshl_b32 {sr(SW)}, {sr(S_WAVE)}, 6")
    e.raw(f"v_lshrrev_b32 {vr(TA)}, {LG}, {vr(LANE)}")                   # row of this lane within an access
    e.raw(f"v_and_b32 {vr(TB)}, {LPR - 1}, {vr(LANE)}")
    e.raw(f"v_lshlrev_b32 {vr(TB)}, 4, {vr(TB)}")                        # byte column of this lane
    e.raw(f"v_add_u32 {vr(GOFF)}, {sr(SW)}, {vr(TA)}")
    e.raw(f"v_mul_lo_u32 {vr(GOFF)}, {vr(GOFF)}, {sr(STEP)}")
    e.raw(f"v_add_u32 {vr(GOFF)}, {vr(GOFF)}, {vr(TB)}")
    e.raw(f"v_lshrrev_b32 {vr(GOFF2)}, 1, {vr(GOFF)}")                   # the same in the bf16 copy
    e.raw(f"s_mul_i32 {sr(SW)}, {sr(S_WAVE)}, {2 * 32 * RSL}")
    e.raw(f"s_add_u32 {sr(SW)}, {sr(SW)}, {sr(S_LDS)}")                  # LDS region of this wavefront (two passes)
    e.raw(f"v_mul_u32_u24 {vr(TA)}, {RSL}, {vr(TA)}")
    e.raw(f"v_add_u32 {vr(TA)}, {vr(TA)}, {vr(TB)}")
    e.raw(f"v_add_u32 {vr(LR)}, {sr(SW)}, {vr(TA)}")
    e.raw(f"v_and_b32 {vr(TA)}, 31, {vr(LANE)}")                         # key of this lane, half of the 32 bytes
    e.raw(f"v_mul_u32_u24 {vr(TA)}, {RSL}, {vr(TA)}")
    e.raw(f"v_lshrrev_b32 {vr(TB)}, 5, {vr(LANE)}")
    e.raw(f"v_lshlrev_b32 {vr(TB)}, 4, {vr(TB)}")
    e.raw(f"v_add_u32 {vr(TA)}, {vr(TA)}, {vr(TB)}")
    e.raw(f"v_add_u32 {vr(LW)}, {sr(SW)}, {vr(TA)}")
    e.raw(f"s_mul_i32 {sr(STEP)}, {sr(STEP)}, {RPI}")                    # bytes between two accesses
    e.raw(f"s_lshr_b32 {sr(STEP2)}, {sr(STEP)}, 1")

    passes = [(nb, which) for nb in range(NKB) for which in ("k", "v")]
    l_var = [e.label(f"epi{v}") for v in range(4)]
    l_end = e.label("epi_end")
    for v in (1, 2, 3):
        e.raw(f"s_cmp_eq_u32 {sr(S_FLAGS)}, {v}")
        e.raw(f"s_cbranch_scc1 {l_var[v]}")

    def body(assign, lowp):
        vm, lgkm = InFlight(e, "vmcnt", 1000), InFlight(e, "lgkmcnt", 12)

        def pointer(ptr, p, bf16=False):
            nb, which = passes[p]
            base = (S_DKLP if which == "k" else S_DVLP) if bf16 else (S_DKPTR if which == "k" else S_DVPTR)
            e.raw(f"s_mov_b64 {sr(ptr, 2)}, {sr(base, 2)}")
            if nb:
                if bf16:
                    e.raw(f"s_lshr_b32 {sr(SW)}, {sr(S_RS32)}, 1")
                e.raw(f"s_add_u32 {sr(ptr)}, {sr(ptr)}, {sr(SW if bf16 else S_RS32)}")
                e.raw(f"s_addc_u32 {sr(ptr + 1)}, {sr(ptr + 1)}, 0")

        def step(ptr, by=STEP):
            e.raw(f"s_add_u32 {sr(ptr)}, {sr(ptr)}, {sr(by)}")
            e.raw(f"s_addc_u32 {sr(ptr + 1)}, {sr(ptr + 1)}, 0")

        def loads(p):
            pointer(PTL, p)
            for n in range(NLD):
                vm.issue(f"global_load_dwordx4 {vr(G(p, n), 4)}, {vr(GOFF)}, {sr(PTL, 2)}", ("ld", p, n))
                step(PTL)

        deep = 1 if lowp else 2                         # passes the HBM reads run ahead (the wait counter holds 63)
        if not assign:
            for p in range(deep):
                loads(p)
        for p, (nb, which) in enumerate(passes):
            accf = ACC_K if which == "k" else ACC_V
            region = 32 * RSL * (p % 2)
            for k in range(4 * DB):
                db, j = divmod(k, 4)
                for i in range(4):
                    e.raw(f"v_accvgpr_read_b32 {vr(W(k) + i)}, {ar(accf(db, nb) + 4 * j + i)}")
                e.raw("s_nop 0")
                lgkm.issue(f"ds_write_b128 {vr(LW)}, {vr(W(k), 4)} offset:{region + 128 * db + 32 * j}", ("w", p, k))
            ahead = min(8, NLD)
            for n in range(ahead):
                lgkm.issue(f"ds_read_b128 {vr(T(n), 4)}, {vr(LR)} offset:{region + n * RPI * RSL}", ("r", p, n))
            pointer(PTS, p)
            if lowp:
                pointer(PTB, p, bf16=True)
            for n in range(NLD):
                lgkm.need(("r", p, n))
                if assign:
                    res = T(n)                          # the value itself is the result
                    if which == "k":
                        for i in range(4):
                            e.raw(f"v_mul_f32 {vr(res + i)}, {sr(S_SCALE)}, {vr(res + i)}")
                else:
                    res = G(p, n)
                    vm.need(("ld", p, n))
                    for i in range(4):
                        if which == "k":
                            e.raw(f"v_fma_f32 {vr(res + i)}, {vr(T(n) + i)}, {sr(S_SCALE)}, {vr(res + i)}")
                        else:
                            e.raw(f"v_add_f32 {vr(res + i)}, {vr(T(n) + i)}, {vr(res + i)}")
                if n + ahead < NLD:
                    m = n + ahead
                    lgkm.issue(f"ds_read_b128 {vr(T(m), 4)}, {vr(LR)} offset:{region + m * RPI * RSL}", ("r", p, m))
                vm.issue(f"global_store_dwordx4 {vr(GOFF)}, {vr(res, 4)}, {sr(PTS, 2)}", ("st", p, n))
                step(PTS)
                if lowp:
                    lo = 192 + 2 * (n % 8)
                    e.raw(f"v_cvt_pk_bf16_f32 {vr(lo)}, {vr(res)}, {vr(res + 1)}")
                    e.raw(f"v_cvt_pk_bf16_f32 {vr(lo + 1)}, {vr(res + 2)}, {vr(res + 3)}")
                    vm.issue(f"global_store_dwordx2 {vr(GOFF2)}, {vr(lo, 2)}, {sr(PTB, 2)}", ("sb", p, n))
                    step(PTB, STEP2)
            if not assign and p + deep < len(passes):   # the registers just stored take the HBM values of a later pass
                loads(p + deep)

    for v in range(4):
        e.raw(l_var[v] + ":")
        body(assign=bool(v & 1), lowp=bool(v & 2))
        if v < 3:
            e.raw(f"s_branch {l_end}")
    e.raw(l_end + ":")


def generate():
    e = Emitter()
    pool = Pool()
    e.comment("---- prologue: stream state")
    for t, s_ in ((T_QPTR, S_QPTR), (T_QHEAD, S_QPTR), (T_DOPTR, S_DOPTR), (T_DOHEAD, S_DOPTR),
                  (T_LSEPTR, S_LSEPTR), (T_LSEHEAD, S_LSEPTR), (T_DLPTR, S_DLPTR), (T_DLHEAD, S_DLPTR),
                  (T_VPTR, S_VPTR)):
        e.raw(f"s_mov_b64 {sr(t, 2)}, {sr(s_, 2)}")
    for t in (T_DBLK, T_DSTEP):
        e.raw(f"s_mov_b32 {sr(t)}, 0")
    e.raw(f"s_mov_b32 {sr(T_REM)}, {sr(S_NSTEPS)}")
    e.raw(f"s_ashr_i32 {sr(T_OHI)}, {sr(S_QOUT)}, 31")     # sign extension of the outer increments
    e.raw(f"s_lshl_b32 {sr(T_M0)}, {sr(S_WAVE)}, 10")
    e.raw(f"s_add_u32 {sr(T_M0)}, {sr(T_M0)}, {sr(S_LDS)}")
    e.raw(f"s_mov_b32 {sr(T_HIMASK)}, 0")
    e.raw(f"s_mov_b32 {sr(T_HIMASK + 1)}, -1")
    e.comment("---- resident K fragments (B operands): key row = lane % 32, elements 16 ks + 8 (lane / 32) .. + 7")
    for nb, krow in ((0, I_KROW0), (1, I_KROW1)):
        for ks in range(KS):
            e.raw(f"global_load_dwordx4 {vr(KF(nb, ks), 4)}, {vr(krow, 2)}, off offset:{32 * ks}")
    e.comment("---- V tile of the workgroup (256 rows) to LDS: instruction 4 j + wave covers rows 16 j + 4 wave .. + 3")
    for j in range(256 * ROW // 4096):
        e.raw(f"s_add_u32 m0, {sr(T_M0)}, {VT + 4096 * j}")
        e.raw("s_nop 0")
        e.raw(f"global_load_lds_dwordx4 {vr(I_VOFF)}, {sr(T_VPTR, 2)}")
        if j < 256 * ROW // 4096 - 1:
            e.raw(f"s_add_u32 {sr(T_VPTR)}, {sr(T_VPTR)}, {sr(S_VRS16)}")
            e.raw(f"s_addc_u32 {sr(T_VPTR + 1)}, {sr(T_VPTR + 1)}, 0")
    e.comment("---- per-lane address registers")
    e.raw(f"v_mov_b32 {vr(QOFF)}, {vr(I_QOFF0)}")
    e.raw(f"v_mov_b32 {vr(DOOFF)}, {vr(I_DOOFF0)}")
    if NDQ == 2:
        e.raw(f"v_mov_b32 {vr(QOFF + 1)}, {vr(I_QOFF1)}")
        e.raw(f"v_mov_b32 {vr(DOOFF + 1)}, {vr(I_DOOFF1)}")
    e.raw(f"v_mov_b32 {vr(STAT_G)}, {vr(I_STAT_G)}")
    e.raw(f"v_mov_b32 {vr(STAT_L)}, {vr(I_STAT_L)}")
    e.raw(f"v_mov_b32 {vr(DKV_OFF)}, {vr(I_DKV)}")
    e.raw(f"v_mov_b32 {vr(NINF)}, 0xff800000")
    # g16 = lds_base + 16 * (lane / 32), from stat_l = lds_base + 4 * lane
    e.raw(f"v_subrev_u32 {vr(TMP)}, {sr(S_LDS)}, {vr(I_STAT_L)}")
    e.raw(f"v_lshrrev_b32 {vr(TMP)}, 7, {vr(TMP)}")
    e.raw(f"v_lshlrev_b32 {vr(TMP)}, 4, {vr(TMP)}")
    e.raw(f"v_add_u32 {vr(G16)}, {sr(S_LDS)}, {vr(TMP)}")
    # x[ks] = xbase + (gf16 ^ (ks << 5));  xv[ks] = x[ks] + V tile + wave * 16384
    e.raw(f"s_lshl_b32 {sr(T_X)}, {sr(S_WAVE)}, {14 if D == 128 else 13}")
    e.raw(f"s_add_u32 {sr(T_X)}, {sr(T_X)}, {VT}")
    for ks in range(KS):
        e.raw(f"v_xor_b32 {vr(TMP)}, {32 * ks}, {vr(I_GF16)}")
        e.raw(f"v_add_u32 {vr(X + ks)}, {vr(I_XBASE)}, {vr(TMP)}")
        e.raw(f"v_add_u32 {vr(XV + ks)}, {sr(T_X)}, {vr(X + ks)}")
    # transpose reads: trlo[db] = trbase + (lf16 ^ (db << 6)), trhi[db] = trbase + 2048 + (lf16 ^ 32 ^ (db << 6))
    for db in range(DB):
        e.raw(f"v_xor_b32 {vr(TMP)}, {64 * db}, {vr(I_LF16)}")
        e.raw(f"v_add_u32 {vr(TRLO + db)}, {vr(I_TRBASE)}, {vr(TMP)}")
        e.raw(f"v_xor_b32 {vr(TMP)}, {(64 * db) ^ 32}, {vr(I_LF16)}")
        e.raw(f"v_add_u32 {vr(TRHI + db)}, {vr(I_TRBASE)}, {vr(TMP)}")
        e.raw(f"v_add_u32 {vr(TRHI + db)}, {8 * ROW}, {vr(TRHI + db)}")
    e.comment("---- blocks 0 and 1 requested; accumulators to zero meanwhile")
    for blk in range(2):
        for grp in request_code(blk, blk):
            for ln in grp:
                e.raw(ln)
        for ln in advance_code():
            e.raw(ln)
    for i in range(256):
        e.raw(f"v_accvgpr_write_b32 {ar(i)}, 0")
    e.comment("statistics of block 0 to LDS stage 0, then block 2 requested (its statistics reuse block 0's registers)")
    e.raw(f"s_waitcnt vmcnt({NREQ})")
    stat_publish(e, 0, 0, "stw")
    e.raw("s_waitcnt lgkmcnt(0)")
    e.ds = []
    for grp in request_code(2, 0):
        for ln in grp:
            e.raw(ln)
    for ln in advance_code():
        e.raw(ln)
    e.raw("s_barrier")

    plans = [plan_reads(e, pool, u, u) for u in range(NS)] + [None]
    # what block 0 of every pass through the loop expects to be in flight: its first reads
    for k in range(-EARLY, 0):
        for fn in plans[0][k]:
            fn()
    e.need("0nd3")              # as at the end of a pass through the loop: the early statistics reads have completed
    l_loop, l_done = e.label("loop"), e.label("done")
    e.raw(l_loop + ":")
    entry = list(e.ds)
    entry_next = pool.next % NPOOL
    for u in range(NS):
        if u == NS - 1:
            plans[NS] = plan_reads(e, pool, 0, NS)      # block 0 of the next pass
        gen_step(e, pool, u, u, plans[u], plans[u + 1])
        e.raw(f"s_sub_u32 {sr(T_REM)}, {sr(T_REM)}, 1")
        e.raw(f"s_cmp_eq_u32 {sr(T_REM)}, 0")
        if u < NS - 1:
            e.raw(f"s_cbranch_scc1 {l_done}")
        else:
            e.raw(f"s_cbranch_scc0 {l_loop}")
    strip = lambda tags: [t.lstrip("0123456789") for t in tags]
    assert strip(e.ds) == strip(entry) and pool.next % NPOOL == entry_next, (e.ds, entry)
    e.raw(l_done + ":")
    e.raw("s_waitcnt vmcnt(0) lgkmcnt(0)")

    epilogue(e)
    return e


def main():
    e = generate()
    clob = [f"v{i}" for i in range(256) if not (IN_V <= i < IN_V + 16)] + [f"a{i}" for i in range(256)]
    clob += [f"s{i}" for i in range(64, 96)]
    write_inc(sys.stdout, "gen_bwd_dkv_asm.py" + (" 64" if D == 64 else ""), "ST_DKV_FAST" + ("64" if D == 64 else ""), e,
              LDS_BYTES, clob)


if __name__ == "__main__":
    main()
