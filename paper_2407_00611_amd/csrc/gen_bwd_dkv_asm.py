#!/usr/bin/env python3
"""Generates the gfx950 assembly of the dK/dV main loop (head_dim 128) as a C string literal.

    python gen_bwd_dkv_asm.py > st_bwd_dkv_asm.inc      (build.py does this before compiling)

The text is the body of ONE `asm volatile` statement in st_bwd_dkv_fast.hip.  The C++ kernel around it
computes addresses and hands them over in pinned registers (see IN_V / IN_S below); everything between
the K-fragment loads and the final read-modify-write of dK / dV is written here with hand-assigned
registers, because the kernel needs all 512 registers of a wavefront (256 accumulators in AGPRs, the
resident K fragments and the score tiles in VGPRs) and a fixed interleave of MFMA, LDS and VALU work.

Work of one workgroup (4 wavefronts): 256 keys of one KV head of one chunk (64 per wavefront), against a
run of 32-query blocks that see every one of those keys (no masking in here; blocks that need a mask go
to the general kernel).  Per block and wavefront, with the MFMA C layout "lane = key column":
    phase 1   S   = Q K^T                       A: Q rows from LDS,        B: resident K fragments
    phase 2   dP' = dO V^T - Delta              A: dO rows from LDS,       B: V rows from LDS, C init: -Delta
              VALU: P = exp2(S c - lse log2e), bf16 pack              (runs under phase 2 / 3 MFMAs)
    phase 3   dV^T += dO^T P                    A: dO^T by LDS transpose reads, B: packed P
              VALU: dS = P dP', bf16 pack (in place)                   (runs under phase 3 / 4 MFMAs)
    phase 4   dK^T += Q^T dS                    A: Q^T by LDS transpose reads,  B: packed dS
Q / dO tiles arrive by direct global->LDS loads into a 4-stage ring, three blocks ahead; the per-row
statistics (lse, Delta) are loaded two blocks ahead into registers, transformed once and written to LDS
by every wavefront (identical values), so that no per-element VALU work is spent on them.
"""
import sys

from st_asmgen import Emitter, ar, sr, vr, write_inc

# ------------------------------------------------------------------------------------------------
# register map
# ------------------------------------------------------------------------------------------------
NKB = 2          # 32-key blocks per wavefront
KS = 8           # contraction steps over head_dim (16 each)
DB = 4           # 32-row blocks of head_dim
NS = 4           # LDS stages of the Q / dO ring
PF = 3           # tiles in flight ahead of the one being computed

def KF(nb, ks): return 4 * (8 * nb + ks)            # v[KF : KF+3]
S0 = 64                                              # S[nb][v]  = v[64 + 16 nb + v]   (later P, fp32)
DP0 = 96                                             # dP[nb][v] = v[96 + 16 nb + v]   (later dS, then packed dS)
P16 = 128                                            # P16[nb][m] = v[128 + 8 nb + 4 m : +3]
NL = 144                                             # nl[v] = -lse(row v) * log2e
ND = 160                                             # nd[v] = -Delta(row v)
POOL0, NPOOL = 176, 10                               # fragment pool, 4 registers each
ST = 216                                             # ST + 2 set + {0: lse, 1: Delta}
TMP = 220                                            # 220..222 temporaries, 223 = -inf
NINF = 223
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
S_QBS, S_QHS, S_DOBS, S_DOHS, S_STATHS, S_NBLK, S_NSTEPS, S_CEXP = 40, 41, 42, 43, 44, 45, 46, 47
S_VPTR, S_VRS16, S_LDS, S_DKPTR, S_DVPTR, S_WAVE, S_RS32, S_SCALE = 48, 50, 51, 52, 54, 56, 57, 58
# scalar temporaries (clobbered)
T_QPTR, T_QHEAD, T_DOPTR, T_DOHEAD = 64, 66, 68, 70
T_LSEPTR, T_LSEHEAD, T_DLPTR, T_DLHEAD = 72, 74, 76, 78
T_DBLK, T_DSTEP, T_SBLK, T_SSTEP, T_REM, T_M0, T_HIMASK, T_X, T_VPTR = 80, 81, 82, 83, 84, 85, 86, 88, 90

def ACC_K(db, nb): return 16 * (2 * db + nb)
def ACC_V(db, nb): return 128 + 16 * (2 * db + nb)

# LDS map (bytes, relative to the kernel's LDS base)
STATS = 0                                            # stage s: nl[32] at 256 s, nd[32] at 256 s + 128
def QT(s): return 1024 + 16384 * s
def DOT(s): return 1024 + 16384 * s + 8192
VT = 1024 + 16384 * NS                               # 256 x 128 bf16 V tile (64 KiB)
LDS_BYTES = VT + 65536

LAT = 3          # MFMA slots between the issue of an LDS read and its first use
BUDGET = 6       # issue units of side work per MFMA slot (an MFMA occupies the pipe for 8 quad-cycles)


def gen_step(e: Emitter, u: int):
    """One 32-query block on LDS stage u (the loop is unrolled NS times so that stage addresses are immediates)."""
    s = u
    qt, dot_, stats = QT(s), DOT(s), STATS + 256 * s
    e.comment(f"================ block on stage {s}")

    # ---- DMA of the tile PF blocks ahead into stage (u + PF) % NS, statistics of the block 2 ahead
    sd = (u + PF) % NS
    for tname, ptr, off, tbase in (("q", T_QPTR, QOFF, QT(sd)), ("do", T_DOPTR, DOOFF, DOT(sd))):
        for j in range(2):
            e.raw(f"s_add_u32 m0, {sr(T_M0)}, {tbase + 4096 * j}")
            e.raw("s_nop 0")
            e.raw(f"global_load_lds_dwordx4 {vr(off + j)}, {sr(ptr, 2)}")
    st_set = u % 2
    e.raw(f"global_load_dword {vr(ST + 2 * st_set)}, {vr(STAT_G)}, {sr(T_LSEPTR, 2)}")
    e.raw(f"global_load_dword {vr(ST + 2 * st_set + 1)}, {vr(STAT_G)}, {sr(T_DLPTR, 2)}")
    gen_advance(e, T_DSTEP, T_DBLK, [(T_QPTR, T_QHEAD, S_QBS, S_QHS), (T_DOPTR, T_DOHEAD, S_DOBS, S_DOHS)])
    gen_advance(e, T_SSTEP, T_SBLK, [(T_LSEPTR, T_LSEHEAD, None, S_STATHS), (T_DLPTR, T_DLHEAD, None, S_STATHS)])

    # ---- the MFMA slots of the block: (phase, operands)
    pool_next = [0]
    frag_reg = {}      # tag -> first register
    frag_last_use = {}  # pool index -> instruction count at its last MFMA use

    pool_owner = {}     # pool slot -> tag
    uses_left = {}      # tag -> MFMAs that still have to read it

    def alloc(tag):
        i = pool_next[0] % NPOOL
        pool_next[0] += 1
        old = pool_owner.get(i)
        assert old is None or uses_left[old] == 0, f"fragment {old} overwritten by {tag} before its last use"
        pool_owner[i] = tag
        uses_left[tag] = 1 if tag.startswith("v") else NKB
        frag_reg[tag] = POOL0 + 4 * i
        return POOL0 + 4 * i

    def use(tag):
        uses_left[tag] -= 1
        return frag_reg[tag]

    # LDS reads by the slot after which they are issued (-1: before the first MFMA)
    reads = {k: [] for k in range(-1, 64)}

    def plan(first_use, fn):
        reads[max(first_use - LAT, -1)].append(fn)

    def rd_nat(tag, tile_imm, ks, xbase=X):
        def f():
            r = alloc(tag)
            e.ds_read(f"ds_read_b128 {vr(r, 4)}, {vr(xbase + ks)} offset:{tile_imm}", tag)
        return f

    def rd_tr(tag, tile_imm, m, db):
        def f():
            r = alloc(tag)
            e.ds_read(f"ds_read_b64_tr_b16 {vr(r, 2)}, {vr(TRLO + db)} offset:{tile_imm + 4096 * m}", tag + "lo")
            e.ds_read(f"ds_read_b64_tr_b16 {vr(r + 2, 2)}, {vr(TRHI + db)} offset:{tile_imm + 4096 * m}", tag)
        return f

    def rd_stat(tag, base_reg, imm):
        def f():
            for j in range(4):
                e.ds_read(f"ds_read_b128 {vr(base_reg + 4 * j, 4)}, {vr(G16)} offset:{imm + 32 * j}", f"{tag}{j}")
        return f

    slots = []
    # phase 1
    for ks in range(KS):
        plan(2 * ks, rd_nat(f"q{ks}", qt, ks))
        for nb in range(NKB):
            slots.append(("S", ks, nb))
    plan(0, rd_stat("nd", ND, stats + 128))
    plan(1, rd_stat("nl", NL, stats))
    # phase 2
    for ks in range(KS):
        base = 16 + 2 * ks
        plan(base, rd_nat(f"do{ks}", dot_, ks))
        for nb in range(NKB):
            plan(base + nb, rd_nat(f"v{nb}_{ks}", 8192 * nb, ks, XV))
            slots.append(("dP", ks, nb))
    # phase 3 / 4
    for ph, tile in (("dV", dot_), ("dK", qt)):
        for m in range(2):
            for db in range(DB):
                base = (32 if ph == "dV" else 48) + 2 * (4 * m + db)
                plan(base, rd_tr(f"{ph}t{m}_{db}", tile, m, db))
                for nb in range(NKB):
                    slots.append((ph, m, db, nb))
    assert len(slots) == 64

    # ---- VALU work: (earliest slot, text, registers written, issue units)
    valu = []
    def S(nb, v): return S0 + 16 * nb + v
    def DP(nb, v): return DP0 + 16 * nb + v
    # VALU-1: P = exp2(S c + nl); pack P.  S[nb] is written by slot 14 + nb; its first reader comes three MFMA issues later.
    for m in range(2):
        for nb in range(NKB):
            early = 17 + nb
            for grp in range(2):
                vs = [8 * m + 4 * grp + i for i in range(4)]
                for v in vs:
                    valu.append((early, f"v_fma_f32 {vr(S(nb, v))}, {vr(S(nb, v))}, {sr(S_CEXP)}, {vr(NL + v)}", (), 1, f"nl{v // 4}"))
                for v in vs:
                    valu.append((early, f"v_exp_f32 {vr(S(nb, v))}, {vr(S(nb, v))}", (), 2, None))
                if grp == 1:
                    for i in range(4):
                        d = P16 + 8 * nb + 4 * m + i
                        a = S(nb, 8 * m + 2 * i)
                        valu.append((early, f"v_cvt_pk_bf16_f32 {vr(d)}, {vr(a)}, {vr(a + 1)}", (d,), 1, None))
    # VALU-2: dS = P dP', packed in place.  dP[nb] is written by slot 30 + nb; same distance.
    for m in range(2):
        for nb in range(NKB):
            early = 33 + nb
            for v in range(8 * m, 8 * m + 8):
                valu.append((early, f"v_mul_f32 {vr(DP(nb, v))}, {vr(S(nb, v))}, {vr(DP(nb, v))}", (), 1, None))
            for i in range(4):
                d = DP(nb, 4 * m + i)
                a = DP(nb, 8 * m + 2 * i)
                valu.append((early, f"v_cvt_pk_bf16_f32 {vr(d)}, {vr(a)}, {vr(a + 1)}", (d,), 1, None))
    vi = [0]
    produced = {}   # register -> True once its packing instruction is out

    def emit_valu(item):
        _, text, writes, units, needtag = item
        if needtag:
            e.need(needtag + "")   # statistics read (tags nl0..nl3)
        e.valu(text, writes)
        for r in writes:
            produced[r] = True
        return units

    def flush_until(regs):
        # the MFMA about to be issued reads packed registers: emit VALU work until they exist
        while not all(produced.get(r) for r in regs):
            assert vi[0] < len(valu), "packed operand never produced"
            emit_valu(valu[vi[0]])
            vi[0] += 1

    for fn in reads[-1]:
        fn()
    for k, sl in enumerate(slots):
        ph = sl[0]
        if ph == "S":
            _, ks, nb = sl
            e.need(f"q{ks}")
            c = "0" if ks == 0 else vr(S0 + 16 * nb, 16)
            e.mfma(vr(S0 + 16 * nb, 16), vr(use(f"q{ks}"), 4), vr(KF(nb, ks), 4), c)
        elif ph == "dP":
            _, ks, nb = sl
            e.need(f"do{ks}")
            e.need(f"v{nb}_{ks}")
            if ks == 0:
                e.need("nd3")
                c = vr(ND, 16)
            else:
                c = vr(DP0 + 16 * nb, 16)
            e.mfma(vr(DP0 + 16 * nb, 16), vr(use(f"do{ks}"), 4), vr(use(f"v{nb}_{ks}"), 4), c)
        else:
            _, m, db, nb = sl
            tag = f"{ph}t{m}_{db}"
            e.need(tag)
            if ph == "dV":
                b0, acc = P16 + 8 * nb + 4 * m, ACC_V(db, nb)
            else:
                b0, acc = DP0 + 16 * nb + 4 * m, ACC_K(db, nb)
            flush_until([b0 + i for i in range(4)] if ph == "dV" else [DP0 + 16 * nb + 4 * m + i for i in range(4)])
            e.mfma(ar(acc, 16), vr(use(tag), 4), vr(b0, 4), ar(acc, 16), breads=[b0 + i for i in range(4)])
        # side work of this slot
        units = 0
        for fn in reads[k]:
            n0 = len(e.ds)
            fn()
            units += len(e.ds) - n0
        while vi[0] < len(valu) and valu[vi[0]][0] <= k and units + valu[vi[0]][3] <= BUDGET:
            units += emit_valu(valu[vi[0]])
            vi[0] += 1
    assert vi[0] == len(valu), f"VALU work left over: {len(valu) - vi[0]}"
    assert all(n == 0 for n in uses_left.values())

    # ---- end of block: the next block's tiles have landed, its statistics go to LDS, everyone syncs
    nxt = (u + 1) % NS
    rs = ST + 2 * ((u + 1) % 2)      # statistics loaded during the previous block
    e.raw("s_waitcnt vmcnt(6)")
    e.valu(f"v_mul_f32 {vr(TMP)}, 0xbfb8aa3b, {vr(rs)}")               # -lse * log2(e)
    e.valu(f"v_xor_b32 {vr(TMP + 1)}, 0x80000000, {vr(rs + 1)}")       # -Delta
    e.valu(f"v_cmp_eq_f32 vcc, 0x7f800000, {vr(TMP)}")                 # lse = -inf (empty row): P must be 0
    e.raw("s_nop 1")
    e.valu(f"v_cndmask_b32 {vr(TMP)}, {vr(TMP)}, {vr(NINF)}, vcc")
    e.valu(f"v_cndmask_b32_e64 {vr(TMP)}, {vr(TMP)}, {vr(TMP + 1)}, {sr(T_HIMASK, 2)}")
    e.raw(f"ds_write_b32 {vr(STAT_L)}, {vr(TMP)} offset:{STATS + 256 * nxt}")
    e.raw("s_waitcnt lgkmcnt(0)")
    e.ds = []
    e.raw("s_barrier")


def gen_advance(e: Emitter, step, blk, ptrs):
    """Move a stream of (pointer, head pointer) pairs to the next block; stays on the last block at the end."""
    l_skip, l_wrap = e.label("skip"), e.label("wrap")
    e.raw(f"s_add_u32 {sr(T_X)}, {sr(step)}, 1")
    e.raw(f"s_cmp_ge_u32 {sr(T_X)}, {sr(S_NSTEPS)}")
    e.raw(f"s_cbranch_scc1 {l_skip}")
    e.raw(f"s_mov_b32 {sr(step)}, {sr(T_X)}")
    e.raw(f"s_add_u32 {sr(blk)}, {sr(blk)}, 1")
    e.raw(f"s_cmp_eq_u32 {sr(blk)}, {sr(S_NBLK)}")
    e.raw(f"s_cbranch_scc1 {l_wrap}")
    for ptr, head, bs, hs in ptrs:
        inc = sr(bs) if bs is not None else "128"
        e.raw(f"s_add_u32 {sr(ptr)}, {sr(ptr)}, {inc}")
        e.raw(f"s_addc_u32 {sr(ptr + 1)}, {sr(ptr + 1)}, 0")
    e.raw(f"s_branch {l_skip}")
    e.raw(l_wrap + ":")
    e.raw(f"s_mov_b32 {sr(blk)}, 0")
    for ptr, head, bs, hs in ptrs:
        e.raw(f"s_add_u32 {sr(head)}, {sr(head)}, {sr(hs)}")
        e.raw(f"s_addc_u32 {sr(head + 1)}, {sr(head + 1)}, 0")
        e.raw(f"s_mov_b64 {sr(ptr, 2)}, {sr(head, 2)}")
    e.raw(l_skip + ":")


def gen_dma_block(e: Emitter, stage):
    for ptr, off, tbase in ((T_QPTR, QOFF, QT(stage)), (T_DOPTR, DOOFF, DOT(stage))):
        for j in range(2):
            e.raw(f"s_add_u32 m0, {sr(T_M0)}, {tbase + 4096 * j}")
            e.raw("s_nop 0")
            e.raw(f"global_load_lds_dwordx4 {vr(off + j)}, {sr(ptr, 2)}")
    gen_advance(e, T_DSTEP, T_DBLK, [(T_QPTR, T_QHEAD, S_QBS, S_QHS), (T_DOPTR, T_DOHEAD, S_DOBS, S_DOHS)])


def gen_stat_load(e: Emitter, st_set):
    e.raw(f"global_load_dword {vr(ST + 2 * st_set)}, {vr(STAT_G)}, {sr(T_LSEPTR, 2)}")
    e.raw(f"global_load_dword {vr(ST + 2 * st_set + 1)}, {vr(STAT_G)}, {sr(T_DLPTR, 2)}")
    gen_advance(e, T_SSTEP, T_SBLK, [(T_LSEPTR, T_LSEHEAD, None, S_STATHS), (T_DLPTR, T_DLHEAD, None, S_STATHS)])


def generate():
    e = Emitter()
    e.comment("---- prologue: stream state")
    for t, s_ in ((T_QPTR, S_QPTR), (T_QHEAD, S_QPTR), (T_DOPTR, S_DOPTR), (T_DOHEAD, S_DOPTR),
                  (T_LSEPTR, S_LSEPTR), (T_LSEHEAD, S_LSEPTR), (T_DLPTR, S_DLPTR), (T_DLHEAD, S_DLPTR),
                  (T_VPTR, S_VPTR)):
        e.raw(f"s_mov_b64 {sr(t, 2)}, {sr(s_, 2)}")
    for t in (T_DBLK, T_DSTEP, T_SBLK, T_SSTEP):
        e.raw(f"s_mov_b32 {sr(t)}, 0")
    e.raw(f"s_mov_b32 {sr(T_REM)}, {sr(S_NSTEPS)}")
    e.comment("c = scale * log2(e) (there is no scalar floating point unit)")
    e.raw(f"v_mov_b32 {vr(TMP)}, 0x3fb8aa3b")
    e.raw(f"v_mul_f32 {vr(TMP)}, {sr(S_SCALE)}, {vr(TMP)}")
    e.raw("s_nop 0")
    e.raw(f"v_readfirstlane_b32 {sr(S_CEXP)}, {vr(TMP)}")
    e.raw(f"s_lshl_b32 {sr(T_M0)}, {sr(S_WAVE)}, 10")
    e.raw(f"s_add_u32 {sr(T_M0)}, {sr(T_M0)}, {sr(S_LDS)}")
    e.raw(f"s_mov_b32 {sr(T_HIMASK)}, 0")
    e.raw(f"s_mov_b32 {sr(T_HIMASK + 1)}, -1")
    e.comment("---- resident K fragments (B operands): key row = lane % 32, elements 16 ks + 8 (lane / 32) .. + 7")
    for nb, krow in ((0, I_KROW0), (1, I_KROW1)):
        for ks in range(KS):
            e.raw(f"global_load_dwordx4 {vr(KF(nb, ks), 4)}, {vr(krow, 2)}, off offset:{32 * ks}")
    e.comment("---- V tile of the workgroup (256 rows) to LDS: instruction 4 j + wave covers rows 16 j + 4 wave .. + 3")
    for j in range(16):
        e.raw(f"s_add_u32 m0, {sr(T_M0)}, {VT + 4096 * j}")
        e.raw("s_nop 0")
        e.raw(f"global_load_lds_dwordx4 {vr(I_VOFF)}, {sr(T_VPTR, 2)}")
        if j < 15:
            e.raw(f"s_add_u32 {sr(T_VPTR)}, {sr(T_VPTR)}, {sr(S_VRS16)}")
            e.raw(f"s_addc_u32 {sr(T_VPTR + 1)}, {sr(T_VPTR + 1)}, 0")
    e.comment("---- per-lane address registers")
    e.raw(f"v_mov_b32 {vr(QOFF)}, {vr(I_QOFF0)}")
    e.raw(f"v_mov_b32 {vr(QOFF + 1)}, {vr(I_QOFF1)}")
    e.raw(f"v_mov_b32 {vr(DOOFF)}, {vr(I_DOOFF0)}")
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
    e.raw(f"s_lshl_b32 {sr(T_X)}, {sr(S_WAVE)}, 14")
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
        e.raw(f"v_add_u32 {vr(TRHI + db)}, 2048, {vr(TRHI + db)}")
    e.comment("---- tiles 0..2 and statistics 0..1 in flight; accumulators to zero meanwhile")
    gen_dma_block(e, 0)
    gen_stat_load(e, 0)          # block k's statistics travel in register set k % 2
    gen_dma_block(e, 1)
    gen_dma_block(e, 2)
    gen_stat_load(e, 1)
    for i in range(256):
        e.raw(f"v_accvgpr_write_b32 {ar(i)}, 0")
    e.comment("statistics of block 0 to LDS stage 0")
    e.raw("s_waitcnt vmcnt(10)")
    rs = ST
    e.raw(f"v_mul_f32 {vr(TMP)}, 0xbfb8aa3b, {vr(rs)}")
    e.raw(f"v_xor_b32 {vr(TMP + 1)}, 0x80000000, {vr(rs + 1)}")
    e.raw(f"v_cmp_eq_f32 vcc, 0x7f800000, {vr(TMP)}")
    e.raw("s_nop 1")
    e.raw(f"v_cndmask_b32 {vr(TMP)}, {vr(TMP)}, {vr(NINF)}, vcc")
    e.raw(f"v_cndmask_b32_e64 {vr(TMP)}, {vr(TMP)}, {vr(TMP + 1)}, {sr(T_HIMASK, 2)}")
    e.raw(f"ds_write_b32 {vr(STAT_L)}, {vr(TMP)} offset:{STATS}")
    e.raw("s_waitcnt lgkmcnt(0)")
    e.raw("s_barrier")

    l_loop, l_done = e.label("loop"), e.label("done")
    e.raw(l_loop + ":")
    for u in range(NS):
        gen_step(e, u)
        e.raw(f"s_sub_u32 {sr(T_REM)}, {sr(T_REM)}, 1")
        e.raw(f"s_cmp_eq_u32 {sr(T_REM)}, 0")
        if u < NS - 1:
            e.raw(f"s_cbranch_scc1 {l_done}")
        else:
            e.raw(f"s_cbranch_scc0 {l_loop}")
    e.raw(l_done + ":")
    e.raw("s_waitcnt vmcnt(0)")

    e.comment("---- epilogue: dk_acc += scale * dK, dv_acc += dV; lane = key row, 4 consecutive d per 16-byte access")
    e.raw("s_nop 7")
    e.raw("s_nop 7")
    for nb in range(NKB):
        if nb == 1:
            e.raw(f"v_add_u32 {vr(DKV_OFF)}, {sr(S_RS32)}, {vr(DKV_OFF)}")
        for which, ptr, accf in (("k", S_DKPTR, ACC_K), ("v", S_DVPTR, ACC_V)):
            for db in range(DB):
                for j in range(4):
                    t = S0 + 4 * (4 * db + j)
                    e.raw(f"global_load_dwordx4 {vr(t, 4)}, {vr(DKV_OFF)}, {sr(ptr, 2)} offset:{128 * db + 32 * j}")
            for db in range(DB):
                for j in range(4):
                    t = S0 + 4 * (4 * db + j)
                    e.raw(f"s_waitcnt vmcnt({15 - (4 * db + j)})" if True else "")
                    for i in range(4):
                        e.raw(f"v_accvgpr_read_b32 {vr(TMP)}, {ar(accf(db, nb) + 4 * j + i)}")
                        e.raw("s_nop 0")
                        if which == "k":
                            e.raw(f"v_fma_f32 {vr(t + i)}, {vr(TMP)}, {sr(S_SCALE)}, {vr(t + i)}")
                        else:
                            e.raw(f"v_add_f32 {vr(t + i)}, {vr(TMP)}, {vr(t + i)}")
            for db in range(DB):
                for j in range(4):
                    t = S0 + 4 * (4 * db + j)
                    e.raw(f"global_store_dwordx4 {vr(DKV_OFF)}, {vr(t, 4)}, {sr(ptr, 2)} offset:{128 * db + 32 * j}")
            e.raw("s_waitcnt vmcnt(0)")
    return e


def main():
    e = generate()
    clob = [f"v{i}" for i in range(256) if not (IN_V <= i < IN_V + 16)] + [f"a{i}" for i in range(256)]
    clob += [f"s{S_CEXP}"] + [f"s{i}" for i in range(64, 92)]
    write_inc(sys.stdout, "gen_bwd_dkv_asm.py", "ST_DKV_FAST", e, LDS_BYTES, clob)


if __name__ == "__main__":
    main()
