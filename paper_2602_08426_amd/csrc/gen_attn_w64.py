#!/usr/bin/env python3
"""Generator of the hand-scheduled row loop of sparse_attn_w64_kernel (gfx950).

Writes prism_attn_w64_body.inc: one inline-asm string that processes ONE (q-head, q-block)
row of the block-sparse attention of Sec. 2 "Block-Sparse Attention" for B = 128, d = 128:
64 queries per wave, 2 waves per workgroup, one wave per SIMD (512 registers per lane).

Why a generator: every K / V^T fragment read from LDS feeds two MFMAs (two 32-query tiles), which
halves the LDS operand traffic of a 32-query wave, and the softmax VALU work of one 64-key
half-step is placed by hand in the shadow of the MFMAs of its neighbours.  That needs ~420 live
registers with the output accumulators and the Q fragments pinned in AGPRs and an explicit
instruction order; both are fixed here rather than left to a register allocator.

Formulation (same as the 32-query kernel): S^T = K Q^T on v_mfma_f32_32x32x16_bf16, O^T += V^T P^T
on v_mfma_f32_32x32x16_f16 (P and the V^T image as fp16); in the accumulator lane l holds query l%32 and keys
8*(r/4) + 4*(l/32) + r%4 (r = 0..15) of a 32-key tile.

Software pipeline over half-steps j (64 keys each, two per listed block):
    iteration j:   MFMA  : PV(j-1)  then  S(j+1)
                   VALU  : softmax(j)                     (in the MFMAs' shadow)
                   copies: K(j+2) -> Kbuf[j&1], V(j) -> Vbuf[j&1]   (global -> LDS, asynchronous)
    end of iteration: wait for this wave's copies, workgroup barrier.
S(j) lives in VGPR bank j&1; softmax(j) turns it into P(j) in place (fp16 pairs in the first 8
registers of every 16-register accumulator), which PV(j) reads as its B operand one iteration
later, before S(j+2) overwrites the bank.

Registers (fixed):
    a[0:127]    O^T accumulators  O[dt][qt] at 16*(2*dt+qt)
    a[128:191]  Q fragments       Q[qt][ks] at 128 + 4*(8*qt+ks)
    v[64:191]   S / P banks       bank p, key tile kt, query tile qt at 64 + 64*p + 16*(2*kt+qt)
    v[192:223]  ring of 8 LDS operand fragments
    v[32:63], v[224:255]  per-lane constants, softmax state, temporaries
    v[0:31] and the SGPRs below s40 are left to the compiler.
"""
from __future__ import annotations

import os
import sys

# ----------------------------------------------------------------------------------------------
# register map
# ----------------------------------------------------------------------------------------------
def O(dt, qt):          # AGPR base of O[dt][qt]
    return 16 * (2 * dt + qt)


def Q(qt, ks):          # AGPR base of Q[qt][ks]
    return 128 + 4 * (8 * qt + ks)


def SB(p, kt, qt):      # VGPR base of S bank p, tile (kt, qt)
    return 64 + 64 * p + 16 * (2 * kt + qt)


FR0 = 192               # fragment ring: 8 slots of 4 VGPRs
N_FR = 8

# per-lane constants / state
V_KOFF = 32             # 8 regs: LDS offsets of the K fragment of k-step ks
V_VOFF = 40             # 4 regs: LDS offsets of the V^T fragment of k-step S
V_CPK = 44              # 8 regs: global offsets of this lane's 8 pieces of a K half-tile copy
V_CPV = 52              # 8 regs: ... of a V^T half-tile copy
V_M = 60                # 2 regs: running max (log2 units) per query tile
V_L = 62                # 2 regs: this lane's share of the running sum
V_T = 224               # 32 temporaries v[224:255]:
#   T+0..5 / T+8..13 softmax of query tile 0 / 1;  T+16..25 prologue / epilogue;  T+26,27 mask
#   thresholds;  T+28 pulled queue position, T+29 its increment (drain .. end of row; the debug dump
#   borrows both);  T+30 list offset;  T+31 -inf
V_ALPHA = V_T + 6       # 2 regs: rescale factor decided by the last softmax
V_IDX = V_T + 14        # 1 reg : list entry loaded two blocks ahead
V_ZERO = V_T + 15       # 1 reg : 0

# scalars (clobbered; inputs arrive in compiler-chosen SGPRs and are copied in the prologue)
S_KRS = 40              # 4: buffer resource of K of this kv head
S_VRS = 44              # 4: buffer resource of the V^T image of this kv head
S_CRS = 48              # 4: buffer resource of this row's list entries
S_CV = 52               # list entry b   (block whose V^T halves are copied / consumed)
S_CK = 53               # list entry b+1 (block whose K halves are copied)
S_B1 = 54               # b + 1
S_N = 55                # entries in the list
S_T0 = 56
S_T1 = 57
S_U = 58
S_CAUSAL = 59
S_HAVE_O = 60
S_WAVE = 61
S_FLAG = 62             # 2+2: per query tile "some lane's max moved past the threshold"
S_TMP = 66              # 2
S_SCALE = 68
S_LDS = 69              # LDS byte address of the tile buffers
S_COFF = 70             # byte offset of entry b+2 in the list
S_T2 = 71
S_KBYTES = 72           # bytes of K of one kv head (records of the K resource)
S_MWAVE = 73            # LDS offset of this wave inside a copy piece pair (wave * 1024)
S_LSE = 74              # 2: lse row base (0 = not requested)
S_QB = 76               # 2
S_OB = 78               # 2
S_VBYTES = 92           # bytes of the V^T image of one kv head (records of the V^T resource)
S_CNT = 94              # 2: address of the pull counter of this workgroup's queue
S_MK = 88               # 2: LDS address of this wave's part of Kbuf[0], Kbuf[1]
S_MV = 90               # 2: ... of Vbuf[0], Vbuf[1]

LDS_K = (0, 16384)      # byte offsets of the K half-tile buffers
LDS_V = (32768, 49152)  # ... and of the V^T half-tile buffers

LOG2E_OVER_SQRT_D = 0x3E0293EE      # log2(e) / sqrt(128) = 0.12751743 as fp32 bits
RESCALE_THRESHOLD = 8.0             # rescale O only when a running max grows by more than 2^8
# P and V^T enter the PV product as fp16.  The running max is kept M_OFFSET below the true one, so
# p = 2^(s - m) reaches 2^(M_OFFSET + RESCALE_THRESHOLD) = 4096 at most (fp16 holds 65504) and a
# probability 2^-36 of the largest one is still a non-zero fp16 value.
M_OFFSET = 4.0


# ----------------------------------------------------------------------------------------------
# instruction records with register tracking (for the hazard check)
# ----------------------------------------------------------------------------------------------
class Ins:
    __slots__ = ("text", "kind", "rd", "wr")

    def __init__(self, text, kind, rd=(), wr=()):
        self.text, self.kind, self.rd, self.wr = text, kind, frozenset(rd), frozenset(wr)


def vr(base, n=1):
    return [("v", base + i) for i in range(n)]


def ar(base, n=1):
    return [("a", base + i) for i in range(n)]


def vtxt(base, n=1):
    return f"v{base}" if n == 1 else f"v[{base}:{base + n - 1}]"


def atxt(base, n=1):
    return f"a{base}" if n == 1 else f"a[{base}:{base + n - 1}]"


def mfma_s(dst, afrag, qreg, first):
    """S tile += K fragment (VGPR) x Q fragment (AGPR)."""
    c = "0" if first else vtxt(dst, 16)
    rd = vr(afrag, 4) + ar(qreg, 4) + ([] if first else vr(dst, 16))
    return Ins(f"v_mfma_f32_32x32x16_bf16 {vtxt(dst, 16)}, {vtxt(afrag, 4)}, {atxt(qreg, 4)}, {c}",
               "mfma", rd, vr(dst, 16))


def mfma_pv(odst, afrag, preg):
    """O tile (AGPR) += V^T fragment (VGPR) x P fragment (VGPR)."""
    rd = vr(afrag, 4) + vr(preg, 4) + ar(odst, 16)
    return Ins(f"v_mfma_f32_32x32x16_f16 {atxt(odst, 16)}, {vtxt(afrag, 4)}, {vtxt(preg, 4)}, {atxt(odst, 16)}",
               "mfma", rd, ar(odst, 16))


def ds_read(dst, addr_reg, offset):
    assert 0 <= offset < 65536
    return Ins(f"ds_read_b128 {vtxt(dst, 4)}, v{addr_reg} offset:{offset}", "lds", vr(addr_reg), vr(dst, 4))


def valu(text, rd=(), wr=(), kind="valu"):
    return Ins(text, kind, rd, wr)


def salu(text):
    return Ins(text, "salu")


def nop(n):
    assert 0 <= n <= 7
    return Ins(f"s_nop {n}", "nop")


def wait_lgkm(n):
    return Ins(f"s_waitcnt lgkmcnt({n})", "wait")


# ----------------------------------------------------------------------------------------------
# pieces of one iteration
# ----------------------------------------------------------------------------------------------
def pv_ops(p):
    """PV(j-1) of an iteration whose softmax bank is p^1... caller passes the bank holding P.
    Returns a list of (lds_read, [mfma, mfma]) groups in issue order."""
    groups = []
    for S in range(4):                       # k-steps of 16 keys inside the 64-key half
        kt, sp = S // 2, S % 2
        for dt in range(4):
            def make(slot, S=S, dt=dt, kt=kt, sp=sp):
                fr = FR0 + 4 * slot
                return [mfma_pv(O(dt, qt), fr, SB(p, kt, qt) + 4 * sp) for qt in range(2)]
            groups.append((("v", S, dt), make))
    return groups


def s_ops(p):
    """S(j+1) into bank p: (lds_read, [mfma, mfma]) groups."""
    groups = []
    for ks in range(8):
        for kt in range(2):
            def make(slot, ks=ks, kt=kt):
                fr = FR0 + 4 * slot
                return [mfma_s(SB(p, kt, qt), fr, Q(qt, ks), ks == 0) for qt in range(2)]
            groups.append((("k", ks, kt), make))
    return groups


def frag_read(desc, slot, kbuf, vbuf):
    kind = desc[0]
    if kind == "k":
        _, ks, kt = desc
        return ds_read(FR0 + 4 * slot, V_KOFF + ks, LDS_K[kbuf] + kt * 8192)
    _, S, dt = desc
    return ds_read(FR0 + 4 * slot, V_VOFF + S, LDS_V[vbuf] + dt * 4096)


def mfma_stream(groups, kbuf, vbuf, depth=6):
    """Orders LDS reads `depth` groups ahead of the MFMAs that consume them; one wait per two
    groups.  Returns (reads to issue up front, list of slots); a slot = the instructions that belong
    together around one MFMA."""
    n = len(groups)
    assert n % 2 == 0 and depth % 2 == 0
    out = []
    pre = [frag_read(groups[i][0], i % N_FR, kbuf, vbuf) for i in range(min(depth, n))]
    issued = len(pre)
    for i, (desc, make) in enumerate(groups):
        m0, m1 = make(i % N_FR)
        slot0 = [m0]
        if i % 2 == 0:
            # fragments i and i + 1 must have arrived: reads younger than i + 1 may be outstanding
            slot0.insert(0, wait_lgkm(issued - (i + 2)))
        slot1 = [m1]
        if issued < n:
            # the ring slot being refilled was consumed N_FR - depth groups ago
            slot1.append(frag_read(groups[issued][0], issued % N_FR, kbuf, vbuf))
            issued += 1
        out.append(slot0)
        out.append(slot1)
    return pre, out


def softmax_ops(p, qt, tag):
    """VALU work of softmax(j) for query tile qt on bank p.  Values of the tile live in the two
    accumulators (kt = 0, 1); P is written in place as fp16 pairs."""
    ops = []
    regs = [SB(p, kt, qt) + r for kt in range(2) for r in range(16)]
    t_mx, t_mc, t_a, t_b = V_T + 8 * qt, V_T + 8 * qt + 1, V_T + 8 * qt + 2, V_T + 8 * qt + 3
    t_s0, t_s1 = V_T + 8 * qt + 4, V_T + 8 * qt + 5
    fl = S_FLAG + 2 * qt
    m, l, al = V_M + qt, V_L + qt, V_ALPHA + qt
    # --- row max over the 32 values of this lane, then with the lane that shares the query
    ops.append(valu(f"v_max3_f32 v{t_mx}, v{regs[0]}, v{regs[1]}, v{regs[2]}", vr(regs[0]) + vr(regs[1]) + vr(regs[2]), vr(t_mx)))
    i = 3
    while i < 32:
        if i + 1 < 32:
            ops.append(valu(f"v_max3_f32 v{t_mx}, v{t_mx}, v{regs[i]}, v{regs[i + 1]}",
                            vr(t_mx) + vr(regs[i]) + vr(regs[i + 1]), vr(t_mx)))
            i += 2
        else:
            ops.append(valu(f"v_max_f32 v{t_mx}, v{t_mx}, v{regs[i]}", vr(t_mx) + vr(regs[i]), vr(t_mx)))
            i += 1
    ops.append(valu(f"v_mov_b32 v{t_mc}, v{t_mx}", vr(t_mx), vr(t_mc)))
    ops.append(valu(f"v_permlane32_swap_b32 v{t_mx}, v{t_mc}", vr(t_mx) + vr(t_mc), vr(t_mx) + vr(t_mc), "lane"))
    ops.append(valu(f"v_max_f32 v{t_mx}, v{t_mx}, v{t_mc}", vr(t_mx) + vr(t_mc), vr(t_mx)))
    # --- m_cand = max(m, mx * scale); move only if it exceeds m + threshold
    ops.append(valu(f"v_fma_f32 v{t_mx}, v{t_mx}, s{S_SCALE}, -{M_OFFSET:.1f}", vr(t_mx), vr(t_mx)))
    ops.append(valu(f"v_max_f32 v{t_mc}, v{m}, v{t_mx}", vr(m) + vr(t_mx), vr(t_mc)))
    ops.append(valu(f"v_add_f32 v{t_a}, 0x{f32_bits(RESCALE_THRESHOLD):08x}, v{m}", vr(m), vr(t_a)))
    ops.append(valu(f"v_cmp_gt_f32 s[{fl}:{fl + 1}], v{t_mc}, v{t_a}", vr(t_mc) + vr(t_a), [("s", fl), ("s", fl + 1)]))
    ops.append(valu(f"v_sub_f32 v{t_b}, v{m}, v{t_mc}", vr(m) + vr(t_mc), vr(t_b)))
    ops.append(valu(f"v_exp_f32 v{t_b}, v{t_b}", vr(t_b), vr(t_b), "trans"))
    ops.append(valu(f"v_cndmask_b32 v{m}, v{m}, v{t_mc}, s[{fl}:{fl + 1}]", vr(m) + vr(t_mc) + [("s", fl)], vr(m)))
    ops.append(valu(f"v_cndmask_b32 v{al}, 1.0, v{t_b}, s[{fl}:{fl + 1}]", vr(t_b) + [("s", fl)], vr(al)))
    # --- p = 2^(s * scale - m), in place; sums in two chains; fp16 pairs in place
    first = [True, True]
    pend = []                                   # exps issued, not yet added / packed
    def flush_one():
        k = pend.pop(0)
        ch = k % 2
        src = regs[k]
        if first[ch]:
            ops.append(valu(f"v_mov_b32 v{t_s0 + ch}, v{src}", vr(src), vr(t_s0 + ch)))
            first[ch] = False
        else:
            ops.append(valu(f"v_add_f32 v{t_s0 + ch}, v{t_s0 + ch}, v{src}", vr(t_s0 + ch) + vr(src), vr(t_s0 + ch)))
        if k % 2 == 1:                          # both members of the pair (k-1, k) have been summed
            kt, r = divmod(k, 16)
            dst = SB(p, kt, qt) + (r - 1) // 2
            ops.append(valu(f"v_cvt_pk_f16_f32 v{dst}, v{regs[k - 1]}, v{regs[k]}",
                            vr(regs[k - 1]) + vr(regs[k]), vr(dst)))
    for k in range(32):
        ops.append(valu(f"v_fma_f32 v{regs[k]}, v{regs[k]}, s{S_SCALE}, -v{m}", vr(regs[k]) + vr(m), vr(regs[k])))
        if k >= 1:
            ops.append(valu(f"v_exp_f32 v{regs[k - 1]}, v{regs[k - 1]}", vr(regs[k - 1]), vr(regs[k - 1]), "trans"))
            pend.append(k - 1)
        if len(pend) > 2:
            flush_one()
    ops.append(valu(f"v_exp_f32 v{regs[31]}, v{regs[31]}", vr(regs[31]), vr(regs[31]), "trans"))
    pend.append(31)
    while pend:
        flush_one()
    # --- l = l * alpha + (sum0 + sum1)
    ops.append(valu(f"v_add_f32 v{t_s0}, v{t_s0}, v{t_s1}", vr(t_s0) + vr(t_s1), vr(t_s0)))
    ops.append(valu(f"v_fma_f32 v{l}, v{l}, v{al}, v{t_s0}", vr(l) + vr(al) + vr(t_s0), vr(l)))
    return ops


def f32_bits(x):
    import struct
    return struct.unpack("<I", struct.pack("<f", x))[0]


S_MASK = 80              # 4 x 2: compare results of the causal mask, used two instructions later


def mask_block(p, hh, label):
    """Causal mask of the diagonal block, applied to bank p before its softmax: key
    64*hh + 32*kt + 8*(r/4) + 4*hf + r%4 is hidden from query 64*wave + 32*qt + l32 when it is
    larger.  A compare result is read by its select no
    sooner than two instructions later (VALU-written SGPR read by a VALU)."""
    T = V_T
    ops = [salu(f"s_cmp_eq_u32 s{S_CV}, s{S_U}"),
           salu(f"s_cselect_b32 s{S_T2}, s{S_CAUSAL}, 0"),
           salu(f"s_cmp_eq_u32 s{S_T2}, 0"),
           salu(f"s_cbranch_scc1 {label}")]
    ops.append(valu(f"v_mov_b32 v{T + 31}, 0xff800000", (), vr(T + 31)))
    # thresholds relative to this half's keys: 64*wave + 32*qt + l32 - 4*hf - 64*hh
    ops += lane_ids(INP, T + 16)
    ops.append(valu(f"v_lshlrev_b32 v{T + 20}, 2, v{T + 18}", vr(T + 18), vr(T + 20)))
    ops.append(valu(f"v_sub_u32 v{T + 20}, v{T + 17}, v{T + 20}", vr(T + 17) + vr(T + 20), vr(T + 20)))
    ops.append(valu(f"v_lshl_add_u32 v{T + 20}, v{T + 19}, 6, v{T + 20}", vr(T + 19) + vr(T + 20), vr(T + 20)))
    for qt in range(2):
        c = 32 * qt - 64 * hh
        ops.append(valu(f"v_add_u32 v{T + 26 + qt}, {lit32(c)}, v{T + 20}", vr(T + 20), vr(T + 26 + qt)))
    todo = [(qt, kt, r) for qt in range(2) for kt in range(2) for r in range(16)]
    def cmp_ins(i):
        qt, kt, r = todo[i]
        c = 32 * kt + 8 * (r // 4) + r % 4
        sp = S_MASK + 2 * (i % 4)
        return valu(f"v_cmp_gt_i32 s[{sp}:{sp + 1}], {c}, v{T + 26 + qt}", vr(T + 26 + qt), [("s", sp), ("s", sp + 1)])
    def sel_ins(i):
        qt, kt, r = todo[i]
        reg = SB(p, kt, qt) + r
        sp = S_MASK + 2 * (i % 4)
        return valu(f"v_cndmask_b32 v{reg}, v{reg}, v{T + 31}, s[{sp}:{sp + 1}]", vr(reg) + vr(T + 31) + [("s", sp), ("s", sp + 1)], vr(reg))
    lead = 3
    for i in range(len(todo) + lead):
        if i < len(todo):
            ops.append(cmp_ins(i))
        if i >= lead:
            ops.append(sel_ins(i - lead))
    ops.append(Ins(f"{label}:", "label"))
    return ops


def lit(c):
    return str(c) if -16 <= c <= 64 else f"0x{c:x}"


def lit32(c):
    return str(c) if -16 <= c <= 64 else f"0x{c & 0xffffffff:x}"


def rescale_block(label):
    """O *= alpha (per query tile), only when the last softmax moved some lane's max and O holds
    something.  O lives in AGPRs: read, multiply, write back in batches of 16."""
    ops = [salu(f"s_or_b64 s[{S_TMP}:{S_TMP + 1}], s[{S_FLAG}:{S_FLAG + 1}], s[{S_FLAG + 2}:{S_FLAG + 3}]"),
           salu(f"s_cselect_b32 s{S_T2}, s{S_HAVE_O}, 0"),
           salu(f"s_cmp_eq_u32 s{S_T2}, 0"),
           salu(f"s_cbranch_scc1 {label}")]
    tmp = V_T + 16                       # 8 temporaries (fragment reads may be in flight)
    for qt in range(2):
        for dt in range(4):
            for half in range(2):
                base = O(dt, qt) + 8 * half
                for r in range(8):
                    ops.append(valu(f"v_accvgpr_read_b32 v{tmp + r}, a{base + r}", ar(base + r), vr(tmp + r)))
                for r in range(8):
                    ops.append(valu(f"v_mul_f32 v{tmp + r}, v{tmp + r}, v{V_ALPHA + qt}", vr(tmp + r) + vr(V_ALPHA + qt), vr(tmp + r)))
                for r in range(8):
                    ops.append(valu(f"v_accvgpr_write_b32 a{base + r}, v{tmp + r}", vr(tmp + r), ar(base + r)))
    ops.append(nop(7))
    ops.append(Ins(f"{label}:", "label"))
    return ops


def copy_k(buf, half, blk_reg, guard_label=None):
    """Asynchronous copy of a K half-tile (64 keys x 128 dims, 16 KB) of block s[blk_reg] into
    Kbuf[buf].  Wave w copies rows 32*w .. 32*w + 31 as 8 pieces of 1 KB (4 rows each); the LDS
    address of piece i is M0 + (i % 4) * 1024 + 16 * lane, so M0 changes twice per tile, and the
    instruction offset that places the piece in LDS is taken out of its global offset V_CPK[i]."""
    ops = []
    if guard_label:
        ops += [salu(f"s_cmp_lt_u32 s{S_B1}, s{S_N}"), salu(f"s_cbranch_scc0 {guard_label}")]
    ops.append(salu(f"s_mov_b32 m0, s{S_MK + buf}"))
    ops.append(salu(f"s_lshl_b32 s{S_T0}, s{blk_reg}, 15"))                   # block * 32 KB
    if half:
        ops.append(salu(f"s_add_u32 s{S_T0}, s{S_T0}, {16384}"))
    for i in range(8):
        if i == 4:
            ops.append(salu(f"s_add_u32 m0, s{S_MK + buf}, 4096"))
            ops.append(nop(0))
        ops.append(Ins(f"buffer_load_dwordx4 v{V_CPK + i}, s[{S_KRS}:{S_KRS + 3}], s{S_T0} offen offset:{(i % 4) * 1024} lds",
                       "vmem", vr(V_CPK + i)))
    if guard_label:
        ops.append(Ins(f"{guard_label}:", "label"))
    return ops


def copy_v(buf, half, blk_reg):
    """Asynchronous copy of a V^T half-tile (128 dims x 64 keys, 16 KB) of block s[blk_reg] into
    Vbuf[buf]: wave w copies dims 64*w .. 64*w + 63 as 8 pieces of 1 KB (8 rows of 128 bytes)."""
    ops = [salu(f"s_mov_b32 m0, s{S_MV + buf}"),
           salu(f"s_lshl_b32 s{S_T1}, s{blk_reg}, 15")]
    if half:
        ops.append(salu(f"s_add_u32 s{S_T1}, s{S_T1}, {128}"))
    else:
        ops.append(nop(0))
    for i in range(8):
        if i == 4:
            ops.append(salu(f"s_add_u32 m0, s{S_MV + buf}, 4096"))
            ops.append(nop(0))
        ops.append(Ins(f"buffer_load_dwordx4 v{V_CPV + i}, s[{S_VRS}:{S_VRS + 3}], s{S_T1} offen offset:{(i % 4) * 1024} lds",
                       "vmem", vr(V_CPV + i)))
    return ops


def load_idx():
    """Entry b+2 of the list (reads past its end return 0 and are never used)."""
    return [valu(f"v_mov_b32 v{V_T + 30}, s{S_COFF}", (), vr(V_T + 30)),
            Ins(f"buffer_load_dword v{V_IDX}, v{V_T + 30}, s[{S_CRS}:{S_CRS + 3}], 0 offen", "vmem",
                vr(V_T + 30), vr(V_IDX))]


def end_of_iteration():
    return [Ins("s_waitcnt vmcnt(0) lgkmcnt(0)", "wait"), Ins("s_barrier", "barrier")]


def interleave(slots, vops):
    """MFMA slots with the VALU ops spread evenly over them (program order kept on both sides)."""
    out = []
    n = len(slots)
    v = list(vops)
    nv = len(v)
    done = 0
    for i, slot in enumerate(slots):
        out += slot
        want = (nv * (i + 1)) // n if n else nv
        while done < want:
            out.append(v[done])
            done += 1
    out += v[done:]
    return out


def zip_streams(a, b):
    out = []
    for i in range(max(len(a), len(b))):
        if i < len(a):
            out.append(a[i])
        if i < len(b):
            out.append(b[i])
    return out


# Tile copies in flight.  Iteration j issues K(j+2) at its start and V(j+1) at its middle; each is
# waited for one and a half iterations later (K(j+1) at the middle of j, V(j) at the end of j), with
# the two younger copies (8 loads each) still in flight.
WAIT_OLDER_COPY = "s_waitcnt vmcnt(16) lgkmcnt(0)"
LEAD_VALU = 12          # side-stream instructions issued between the up-front LDS reads and the first MFMA


HOLD = 2                # fragment groups whose MFMAs are issued behind the next barrier
DEPTH = 6               # fragment groups read ahead of their MFMAs
INCOMING_SIDE = 14      # side instructions issued beside the held-back MFMAs (the copy's issue)


def sync_point(which):
    """Wait for this wave's older tile copy, then the workgroup barrier.  The timing experiments
    (PRISM_W64_EXPERIMENT, wrong results by construction, never part of the product build) leave
    out the barrier ("nobar_mid", "nobar_end") or the wait for the copies ("nowait")."""
    ops = [Ins("s_waitcnt lgkmcnt(0)" if "nowait" in EXPERIMENT else WAIT_OLDER_COPY, "wait")]
    if f"nobar_{which}" not in EXPERIMENT:
        ops.append(Ins("s_barrier", "barrier"))
    return ops


def held_s_mfmas(bank):
    """MFMAs of the last HOLD fragment groups of an S phase into `bank` (their fragments sit in
    the last ring slots: every phase has 16 groups, so group 14 + i is in slot 6 + i)."""
    out = []
    groups = s_ops(bank)
    for i in range(16 - HOLD, 16):
        out += groups[i][1](i % N_FR)
    return out


def segment(groups, g0, kbuf, vbuf):
    """Fragment reads and MFMA slots of one phase, all but its last HOLD groups.
    Returns (reads to issue up front, slots, MFMAs held back)."""
    n = len(groups)
    pre = [frag_read(groups[i][0], (g0 + i) % N_FR, kbuf, vbuf) for i in range(DEPTH)]
    issued = DEPTH
    slots = []
    for i in range(n - HOLD):
        m0, m1 = groups[i][1]((g0 + i) % N_FR)
        s0 = [m0]
        if i % 2 == 0:
            s0.insert(0, wait_lgkm(issued - (i + 2)))
        s1 = [m1]
        if issued < n:
            s1.append(frag_read(groups[issued][0], (g0 + issued) % N_FR, kbuf, vbuf))
            issued += 1
        slots += [s0, s1]
    assert issued == n
    held = []
    for i in range(n - HOLD, n):
        held += groups[i][1]((g0 + i) % N_FR)
    return pre, slots, held


def iteration(p, hh, do_pv, do_s, incoming, uid, sequential=False):
    """One iteration j with softmax bank p = j & 1 and half hh = j & 1 of its block.
    do_pv: PV(j-1) exists; do_s: S(j+1) exists; incoming: the previous iteration left the last
    MFMAs of S(j) to be issued here (behind its closing barrier).
        start : every wave is done reading K(j) and V(j-1) has landed
                [last MFMAs of S(j)]  copy K(j+2) -> Kbuf[p]      (half hh of block b+1)
                PV(j-1) from Vbuf[q], first half of softmax(j)
        middle: wait K(j+1), barrier: every wave is done reading V(j-1)
                [last MFMAs of PV(j-1)]  copy V(j+1) -> Vbuf[q]   (half 1 of block b / half 0 of b+1)
                S(j+1) from Kbuf[q] into bank q, second half of softmax(j)
        end   : wait V(j), barrier
    The MFMAs held back across a barrier already have their fragments in registers; they keep the
    matrix pipe busy while the first fragments of the next phase travel from LDS.
    Past the end of the list the K / V^T resource is given zero records, so those copies touch no
    memory (the number of loads in flight stays a compile-time fact)."""
    q = p ^ 1
    vops = zip_streams(softmax_ops(p, 0, uid), softmax_ops(p, 1, uid))
    if "nosoft" in EXPERIMENT:
        vops = []
    n_a = len(vops) // 2 if (do_pv and do_s) else (len(vops) if do_pv else 0)
    copy_a, copy_b = [], []
    if "nocopy" not in EXPERIMENT:
        copy_a += [salu(f"s_cmp_lt_u32 s{S_B1}, s{S_N}"),
                   salu(f"s_cselect_b32 s{S_KRS + 2}, s{S_KBYTES}, 0")]
        copy_a += copy_k(p, hh, S_CK)
        if hh == 1:
            copy_b += [salu(f"s_cmp_lt_u32 s{S_B1}, s{S_N}"),
                       salu(f"s_cselect_b32 s{S_VRS + 2}, s{S_VBYTES}, 0")]
            copy_b += copy_v(q, 0, S_CK)
        else:
            copy_b += copy_v(q, 1, S_CV)
    if hh == 0:
        copy_a += load_idx()
    inc = held_s_mfmas(p) if incoming else []

    ops = []
    # ---- first phase
    if do_pv:
        pre, slots, held1 = segment(pv_ops(q), 0, q, q)
        ops += pre
        ops += interleave([[m] for m in inc], copy_a) if inc else copy_a
        ops += rescale_block(f"Lnoresc_{uid}")
        ops += mask_block(p, hh, f"Lnomask_{uid}")
        ops += interleave(slots, vops[:n_a])
    else:
        assert not inc
        held1 = []
        ops += copy_a
        ops += mask_block(p, hh, f"Lnomask_{uid}")
    ops += sync_point("mid")
    # ---- second phase
    if do_s:
        pre, slots, held2 = segment(s_ops(q), 16 if do_pv else 0, q, q)
        ops += pre
        if held1:
            ops += interleave([[m] for m in held1], copy_b)
            ops += interleave(slots, vops[n_a:])
        else:
            ops += interleave(slots, copy_b + vops[n_a:])
    else:
        held2 = []
        ops += interleave([[m] for m in held1], copy_b + vops[n_a:])
    if uid in ("o0", "oZ"):
        ops.append(salu(f"s_mov_b32 s{S_HAVE_O}, 1"))
    ops += sync_point("end")
    if hh == 1:
        # next block: entry b+1 becomes b, the entry loaded two ahead becomes b+1
        ops += [salu(f"s_mov_b32 s{S_CV}, s{S_CK}"),
                valu(f"v_readfirstlane_b32 s{S_CK}, v{V_IDX}", vr(V_IDX), [("s", S_CK)], "lane"),
                salu(f"s_add_u32 s{S_B1}, s{S_B1}, 1"),
                salu(f"s_add_u32 s{S_COFF}, s{S_COFF}, 4")]
    return ops


def pull_next_row():
    """Lane 0 of wave 0 takes the workgroup's next position in its queue (returning atomic add on the
    queue's pull counter); the answer travels while the last PV and the epilogue run and is handed
    to the C++ loop in the asm block's output operand.  Pulling only now, when the row is almost
    done, keeps the rows that an XCD's workgroups work on at any time neighbours in the queue, i.e.
    neighbouring q-blocks of one head, whose lists share tiles in the L2."""
    T = V_T
    return [salu(f"s_cmp_lg_u32 s{S_WAVE}, 0"),
            salu("s_cbranch_scc1 Lnopull"),
            salu(f"s_mov_b64 s[{S_TMP}:{S_TMP + 1}], exec"),
            salu("s_mov_b64 exec, 1"),
            valu(f"v_mov_b32 v{T + 29}, 1", (), vr(T + 29)),
            Ins(f"global_atomic_add v{T + 28}, v{V_ZERO}, v{T + 29}, s[{S_CNT}:{S_CNT + 1}] sc0", "vmem",
                vr(V_ZERO) + vr(T + 29), vr(T + 28)),
            salu(f"s_mov_b64 exec, s[{S_TMP}:{S_TMP + 1}]"),
            Ins("Lnopull:", "label")]


def drain(p_bank):
    """PV of the last half-step (its P is in bank p_bank, its V^T half in Vbuf[p_bank])."""
    pre, slots = mfma_stream(pv_ops(p_bank), p_bank, p_bank)
    ops = pull_next_row() + rescale_block("Lnoresc_drain") + pre
    for s in slots:
        ops += s
    ops += [nop(7), nop(7), nop(7)]
    return ops


# ----------------------------------------------------------------------------------------------
# prologue / epilogue of a row
# ----------------------------------------------------------------------------------------------
def lane_ids(inp, T):
    """T+0 = lane, T+1 = lane & 31, T+2 = lane >> 5, T+3 = wave, from the thread index."""
    t = inp["t"]
    return [valu(f"v_and_b32 v{T}, 63, {t}", (), vr(T)),
            valu(f"v_and_b32 v{T + 1}, 31, {t}", (), vr(T + 1)),
            valu(f"v_lshrrev_b32 v{T + 2}, 5, v{T}", vr(T), vr(T + 2)),
            valu(f"v_lshrrev_b32 v{T + 3}, 6, {t}", (), vr(T + 3))]


def prologue(inp):
    """inp: dict name -> inline-asm operand text ("%3", ...)."""
    T = V_T
    ops = []
    a = ops.append
    # scalars
    a(salu(f"s_mov_b32 s{S_N}, {inp['n']}"))
    a(salu(f"s_mov_b32 s{S_U}, {inp['u']}"))
    a(salu(f"s_mov_b32 s{S_CAUSAL}, {inp['causal']}"))
    a(salu(f"s_mov_b32 s{S_LDS}, {inp['lds']}"))
    a(salu(f"s_mov_b64 s[{S_LSE}:{S_LSE + 1}], {inp['lse']}"))
    a(salu(f"s_mov_b64 s[{S_QB}:{S_QB + 1}], {inp['q']}"))
    a(salu(f"s_mov_b64 s[{S_OB}:{S_OB + 1}], {inp['o']}"))
    a(salu(f"s_mov_b32 s{S_SCALE}, 0x{LOG2E_OVER_SQRT_D:08x}"))
    a(salu(f"s_mov_b32 s{S_HAVE_O}, 0"))
    a(salu(f"s_mov_b64 s[{S_FLAG}:{S_FLAG + 1}], 0"))
    a(salu(f"s_mov_b64 s[{S_FLAG + 2}:{S_FLAG + 3}], 0"))
    a(salu(f"s_mov_b64 s[{S_CNT}:{S_CNT + 1}], {inp['cnt']}"))
    a(salu(f"s_mov_b32 s{S_KBYTES}, {inp['kbytes']}"))
    a(salu(f"s_mov_b32 s{S_VBYTES}, {inp['vbytes']}"))
    for rs, ptr, nbytes in ((S_KRS, inp["k"], inp["kbytes"]), (S_VRS, inp["vt"], inp["vbytes"])):
        a(salu(f"s_mov_b64 s[{rs}:{rs + 1}], {ptr}"))
        a(salu(f"s_and_b32 s{rs + 1}, s{rs + 1}, 0xffff"))
        a(salu(f"s_mov_b32 s{rs + 2}, {nbytes}"))
        a(salu(f"s_mov_b32 s{rs + 3}, 0x00020000"))
    a(salu(f"s_mov_b64 s[{S_CRS}:{S_CRS + 1}], {inp['col']}"))
    a(salu(f"s_and_b32 s{S_CRS + 1}, s{S_CRS + 1}, 0xffff"))
    a(salu(f"s_lshl_b32 s{S_CRS + 2}, s{S_N}, 2"))
    a(salu(f"s_mov_b32 s{S_CRS + 3}, 0x00020000"))
    # per-lane constants from the thread index
    ops += lane_ids(inp, T)
    a(nop(1))
    a(valu(f"v_readfirstlane_b32 s{S_WAVE}, v{T + 3}", vr(T + 3), [("s", S_WAVE)], "lane"))
    a(valu(f"v_mov_b32 v{V_ZERO}, 0", (), vr(V_ZERO)))
    # K copy pieces: piece i of this wave = rows 32*wave + 4*i .. + 3 of the half-tile; LDS slot
    # (row, c') holds global chunk c' ^ (row & 15)
    a(valu(f"v_lshrrev_b32 v{T + 4}, 4, v{T}", vr(T), vr(T + 4)))              # lane >> 4  (0..3)
    a(valu(f"v_and_b32 v{T + 5}, 15, v{T}", vr(T), vr(T + 5)))                 # lane & 15
    a(valu(f"v_lshlrev_b32 v{T + 6}, 13, v{T + 3}", vr(T + 3), vr(T + 6)))     # wave * 8192
    a(valu(f"v_lshl_add_u32 v{T + 6}, v{T + 4}, 8, v{T + 6}", vr(T + 4) + vr(T + 6), vr(T + 6)))
    for i in range(4):
        a(valu(f"v_or_b32 v{T + 7}, {4 * i}, v{T + 4}", vr(T + 4), vr(T + 7)))
        a(valu(f"v_xor_b32 v{T + 7}, v{T + 7}, v{T + 5}", vr(T + 7) + vr(T + 5), vr(T + 7)))
        a(valu(f"v_lshl_add_u32 v{V_CPK + i}, v{T + 7}, 4, v{T + 6}", vr(T + 7) + vr(T + 6), vr(V_CPK + i)))
        a(valu(f"v_add_u32 v{V_CPK + 4 + i}, 0x1000, v{V_CPK + i}", vr(V_CPK + i), vr(V_CPK + 4 + i)))
    # V^T copy pieces: piece i = rows 64*wave + 8*i .. + 7 (128 bytes each in LDS, 256 in the
    # image); LDS slot (row, c') holds chunk c' ^ ((row >> 1) & 7) of the row's half
    a(valu(f"v_lshrrev_b32 v{T + 5}, 3, v{T}", vr(T), vr(T + 5)))              # lane >> 3
    a(valu(f"v_and_b32 v{T + 7}, 7, v{T}", vr(T), vr(T + 7)))                  # lane & 7
    a(valu(f"v_lshlrev_b32 v{T + 6}, 14, v{T + 3}", vr(T + 3), vr(T + 6)))     # wave * 16384
    a(valu(f"v_lshl_add_u32 v{T + 6}, v{T + 5}, 8, v{T + 6}", vr(T + 5) + vr(T + 6), vr(T + 6)))
    for e in range(2):
        a(valu(f"v_or_b32 v{T + 16 + e}, {4 * e}, v{T + 4}", vr(T + 4), vr(T + 16 + e)))
        a(valu(f"v_xor_b32 v{T + 16 + e}, v{T + 16 + e}, v{T + 7}", vr(T + 16 + e) + vr(T + 7), vr(T + 16 + e)))
        a(valu(f"v_lshl_add_u32 v{T + 16 + e}, v{T + 16 + e}, 4, v{T + 6}", vr(T + 16 + e) + vr(T + 6), vr(T + 16 + e)))
    for i in range(8):
        c = i * 2048 - (i % 4) * 1024
        a(valu(f"v_add_u32 v{V_CPV + i}, {lit(c)}, v{T + 16 + (i & 1)}", vr(T + 16 + (i & 1)), vr(V_CPV + i)))
    a(salu(f"s_lshl_b32 s{S_MWAVE}, s{S_WAVE}, 13"))
    a(salu(f"s_add_u32 s{S_MWAVE}, s{S_MWAVE}, s{S_LDS}"))
    for b in range(2):
        a(salu(f"s_add_u32 s{S_MK + b}, s{S_MWAVE}, {LDS_K[b]}" if LDS_K[b] else f"s_mov_b32 s{S_MK + b}, s{S_MWAVE}"))
        a(salu(f"s_add_u32 s{S_MV + b}, s{S_MWAVE}, {LDS_V[b]}"))
    # K(0) -> Kbuf[0], K(1) -> Kbuf[1]: both halves of the first listed block (its index comes with
    # the row's queue entry, so the copies start before anything else is loaded)
    a(salu(f"s_mov_b32 s{S_CV}, {inp['c0']}"))
    ops += copy_k(0, 0, S_CV)
    ops += copy_k(1, 1, S_CV)
    ops += copy_v(0, 0, S_CV)
    # list entry 1 (reads as 0 when the list has one entry; it is then unused)
    a(Ins(f"buffer_load_dword v{V_IDX}, v{V_ZERO}, s[{S_CRS}:{S_CRS + 3}], 0 offen offset:4", "vmem", vr(V_ZERO), vr(V_IDX)))
    # Q fragments: row 32*qt + l32 of this wave's 64 rows, dims 16*ks + 8*hf .. + 7; through the
    # (idle) S bank 0 into AGPRs; O = 0 while they travel
    a(valu(f"v_lshlrev_b32 v{T + 5}, 8, v{T + 1}", vr(T + 1), vr(T + 5)))
    a(valu(f"v_lshl_add_u32 v{T + 21}, v{T + 2}, 4, v{T + 5}", vr(T + 2) + vr(T + 5), vr(T + 21)))
    a(valu(f"v_add_u32 v{T + 22}, 0x2000, v{T + 21}", vr(T + 21), vr(T + 22)))
    for qt in range(2):
        for ks in range(8):
            dst = SB(0, 0, 0) + 4 * (8 * qt + ks)
            a(Ins(f"global_load_dwordx4 {vtxt(dst, 4)}, v{T + 21 + qt}, s[{S_QB}:{S_QB + 1}] offset:{ks * 32}",
                  "vmem", vr(T + 21 + qt), vr(dst, 4)))
    # LDS read offsets of the MFMA operand fragments
    a(valu(f"v_and_b32 v{T + 4}, 15, v{T + 1}", vr(T + 1), vr(T + 4)))   # l32 & 15
    a(valu(f"v_lshl_add_u32 v{T + 5}, v{T + 1}, 8, s{S_LDS}", vr(T + 1), vr(T + 5)))  # l32 * 256 + LDS base
    for ks in range(8):
        a(valu(f"v_or_b32 v{T + 6}, {2 * ks}, v{T + 2}", vr(T + 2), vr(T + 6)))
        a(valu(f"v_xor_b32 v{T + 6}, v{T + 6}, v{T + 4}", vr(T + 6) + vr(T + 4), vr(T + 6)))
        a(valu(f"v_lshl_add_u32 v{V_KOFF + ks}, v{T + 6}, 4, v{T + 5}", vr(T + 6) + vr(T + 5), vr(V_KOFF + ks)))
    a(valu(f"v_bfe_u32 v{T + 4}, v{T + 1}, 1, 3", vr(T + 1), vr(T + 4)))   # (l32 >> 1) & 7
    a(valu(f"v_lshl_add_u32 v{T + 5}, v{T + 1}, 7, s{S_LDS}", vr(T + 1), vr(T + 5)))  # l32 * 128 + LDS base
    for S in range(4):
        a(valu(f"v_or_b32 v{T + 6}, {2 * S}, v{T + 2}", vr(T + 2), vr(T + 6)))
        a(valu(f"v_xor_b32 v{T + 6}, v{T + 6}, v{T + 4}", vr(T + 6) + vr(T + 4), vr(T + 6)))
        a(valu(f"v_lshl_add_u32 v{V_VOFF + S}, v{T + 6}, 4, v{T + 5}", vr(T + 6) + vr(T + 5), vr(V_VOFF + S)))
    # softmax state
    for qt in range(2):
        a(valu(f"v_mov_b32 v{V_M + qt}, 0xff800000", (), vr(V_M + qt)))
        a(valu(f"v_mov_b32 v{V_L + qt}, 0", (), vr(V_L + qt)))
        a(valu(f"v_mov_b32 v{V_ALPHA + qt}, 1.0", (), vr(V_ALPHA + qt)))
    for r in range(128):
        a(valu(f"v_accvgpr_write_b32 a{r}, 0", (), ar(r)))
    a(Ins("s_waitcnt vmcnt(0)", "wait"))
    for i in range(64):
        a(valu(f"v_accvgpr_write_b32 a{128 + i}, v{SB(0, 0, 0) + i}", vr(SB(0, 0, 0) + i), ar(128 + i)))
    a(valu(f"v_readfirstlane_b32 s{S_CK}, v{V_IDX}", vr(V_IDX), [("s", S_CK)], "lane"))
    a(salu(f"s_mov_b32 s{S_B1}, 1"))
    a(salu(f"s_mov_b32 s{S_COFF}, 8"))
    a(nop(4))
    ops += end_of_iteration()
    # S(0) into bank 0
    pre, slots = mfma_stream(s_ops(0), 0, 0)
    ops += pre
    for sl in slots:
        ops += sl
    ops += [nop(7), nop(7), nop(7)]
    ops += end_of_iteration()          # iteration 0 refills Kbuf[0]: every wave is done reading it
    return ops


def epilogue():
    """O = O^T / l as bf16 rows, lse = (m + log2 l) ln 2 (the offset of m cancels: l is the sum
    of 2^(s - m) with the same m)."""
    T = V_T
    ops = []
    a = ops.append
    # row offsets of this lane: O row (32*qt + l32) * 256 + hf * 8 bytes, lse (32*qt + l32) * 4
    ops += lane_ids(INP, T)
    a(valu(f"v_lshlrev_b32 v{T + 5}, 8, v{T + 1}", vr(T + 1), vr(T + 5)))
    a(valu(f"v_lshl_add_u32 v{T + 21}, v{T + 2}, 3, v{T + 5}", vr(T + 2) + vr(T + 5), vr(T + 21)))
    a(valu(f"v_add_u32 v{T + 22}, 0x2000, v{T + 21}", vr(T + 21), vr(T + 22)))
    a(valu(f"v_lshlrev_b32 v{T + 23}, 2, v{T + 1}", vr(T + 1), vr(T + 23)))
    a(valu(f"v_add_u32 v{T + 24}, 128, v{T + 23}", vr(T + 23), vr(T + 24)))
    for qt in range(2):
        lt, inv = T + 16 + qt, T + 18 + qt
        a(valu(f"v_mov_b32 v{T + 20}, v{V_L + qt}", vr(V_L + qt), vr(T + 20)))
        a(valu(f"v_mov_b32 v{lt}, v{V_L + qt}", vr(V_L + qt), vr(lt)))
        a(nop(1))
        a(valu(f"v_permlane32_swap_b32 v{lt}, v{T + 20}", vr(lt) + vr(T + 20), vr(lt) + vr(T + 20), "lane"))
        a(nop(1))
        a(valu(f"v_add_f32 v{lt}, v{lt}, v{T + 20}", vr(lt) + vr(T + 20), vr(lt)))
        a(valu(f"v_rcp_f32 v{inv}, v{lt}", vr(lt), vr(inv), "trans"))
        a(nop(3))
    for qt in range(2):
        inv = T + 18 + qt
        for dt in range(4):
            base = O(dt, qt)
            for r in range(16):
                a(valu(f"v_accvgpr_read_b32 v{FR0 + r}, a{base + r}", ar(base + r), vr(FR0 + r)))
            for r in range(16):
                a(valu(f"v_mul_f32 v{FR0 + r}, v{FR0 + r}, v{inv}", vr(FR0 + r) + vr(inv), vr(FR0 + r)))
            st = FR0 + 16 + 8 * (dt & 1)                    # two staging sets, used alternately
            for r in range(0, 16, 2):
                a(valu(f"v_cvt_pk_bf16_f32 v{st + r // 2}, v{FR0 + r}, v{FR0 + r + 1}",
                       vr(FR0 + r) + vr(FR0 + r + 1), vr(st + r // 2)))
            for g4 in range(4):
                a(Ins(f"global_store_dwordx2 v{T + 21 + qt}, {vtxt(st + 2 * g4, 2)}, s[{S_OB}:{S_OB + 1}] offset:{dt * 64 + g4 * 16}",
                      "vmem", vr(T + 21 + qt) + vr(st + 2 * g4, 2)))
    a(salu(f"s_cmp_eq_u64 s[{S_LSE}:{S_LSE + 1}], 0"))
    a(salu("s_cbranch_scc1 Lnolse"))
    for qt in range(2):
        lt = T + 16 + qt
        a(valu(f"v_log_f32 v{lt}, v{lt}", vr(lt), vr(lt), "trans"))
        a(nop(3))
        a(valu(f"v_add_f32 v{lt}, v{lt}, v{V_M + qt}", vr(lt) + vr(V_M + qt), vr(lt)))
        a(valu(f"v_mul_f32 v{lt}, 0x3f317218, v{lt}", vr(lt), vr(lt)))
        a(Ins(f"global_store_dword v{T + 23 + qt}, v{lt}, s[{S_LSE}:{S_LSE + 1}]", "vmem", vr(T + 23 + qt) + vr(lt)))
    a(Ins("Lnolse:", "label"))
    a(Ins("s_waitcnt vmcnt(0)", "wait"))
    return ops


# ----------------------------------------------------------------------------------------------
# debugging aid (never part of a product build): dump registers to the buffer whose address came in
# as the lse pointer, as dbg[i][t] (i = position in `regs`, t = thread 0..127), then leave the row
# ----------------------------------------------------------------------------------------------
def dump_and_exit(regs, inp):
    T = V_T
    ops = [nop(7), nop(7), nop(7),
           valu(f"v_and_b32 v{T + 29}, 63, {inp['t']}", (), vr(T + 29)),
           valu(f"v_lshlrev_b32 v{T + 29}, 2, v{T + 29}", vr(T + 29), vr(T + 29))]
    for kind, r in regs:
        if kind == "a":
            ops.append(valu(f"v_accvgpr_read_b32 v{T + 28}, a{r}", ar(r), vr(T + 28)))
            ops.append(nop(1))
            src = T + 28
        else:
            src = r
        ops.append(Ins(f"global_store_dword v{T + 29}, v{src}, s[{S_LSE}:{S_LSE + 1}]", "vmem", vr(T + 29) + vr(src)))
        ops.append(salu(f"s_add_u32 s{S_LSE}, s{S_LSE}, 512"))
        ops.append(salu(f"s_addc_u32 s{S_LSE + 1}, s{S_LSE + 1}, 0"))
        ops.append(Ins("s_waitcnt vmcnt(0)", "wait"))
    ops.append(salu("s_branch Lrow_done"))
    return ops


DUMP = os.environ.get("PRISM_W64_DUMP", "")
# timing experiments (wrong results, same control flow): leave out the tile copies of the steady-state
# iterations / the softmax arithmetic
EXPERIMENT = os.environ.get("PRISM_W64_EXPERIMENT", "")


# ----------------------------------------------------------------------------------------------
# whole row
# ----------------------------------------------------------------------------------------------
def row_program(inp, sequential=False):
    ops = prologue(inp)
    a = ops.append
    if DUMP == "LDS":
        ops.append(valu(f"v_and_b32 v{V_T + 27}, 63, {inp['t']}", (), vr(V_T + 27)))
        ops.append(valu(f"v_lshlrev_b32 v{V_T + 27}, 4, v{V_T + 27}", vr(V_T + 27), vr(V_T + 27)))
        for kk in range(64):
            ops.append(Ins(f"ds_read_b32 v{64 + kk}, v{V_T + 27} offset:{kk * 1024}", "lds", vr(V_T + 27), vr(64 + kk)))
        ops.append(Ins("s_waitcnt lgkmcnt(0)", "wait"))
        for i, sreg in enumerate((S_WAVE, S_MWAVE, S_LDS, S_T1, S_CV, S_N, S_U)):
            ops.append(valu(f"v_mov_b32 v{128 + i}, s{sreg}", (), vr(128 + i)))
        ops.append(valu(f"v_mov_b32 v{128 + 8}, {inp['t']}", (), vr(128 + 8)))
        ops += dump_and_exit([("v", 64 + i) for i in range(64 + 9)], inp)
    if DUMP == "S0":
        ops += [ds_read(FR0, V_KOFF, LDS_K[0]), ds_read(FR0 + 4, V_KOFF + 1, LDS_K[0] + 8192),
                Ins("s_waitcnt lgkmcnt(0)", "wait")]
        ops += dump_and_exit([("v", 64 + i) for i in range(64)] + [("a", 128 + i) for i in range(64)] +
                             [("v", FR0 + i) for i in range(8)] + [("v", V_KOFF + i) for i in range(16)] +
                             [("v", V_QOFF), ("v", V_QOFF + 1)], inp)
    # block 0, even iteration: no PV yet
    ops += iteration(0, 0, False, True, False, "e0", sequential)
    if DUMP == "I0":
        ops += dump_and_exit([("v", 64 + i) for i in range(128)] +
                             [("v", V_M), ("v", V_M + 1), ("v", V_L), ("v", V_L + 1), ("v", V_ALPHA), ("v", V_ALPHA + 1)], inp)
    a(salu(f"s_cmp_eq_u32 s{S_N}, 1"))
    a(salu("s_cbranch_scc1 Lodd_last"))
    ops += iteration(1, 1, True, True, True, "o0", sequential)
    a(Ins("Lloop:", "label"))
    # here S_B1 = (block index b of the coming even iteration) + 1
    a(salu(f"s_cmp_eq_u32 s{S_B1}, s{S_N}"))
    a(salu("s_cbranch_scc1 Leven_last"))
    ops += iteration(0, 0, True, True, True, "eL", sequential)
    ops += iteration(1, 1, True, True, True, "oL", sequential)
    a(salu("s_branch Lloop"))
    a(Ins("Leven_last:", "label"))
    ops += iteration(0, 0, True, True, True, "eZ", sequential)
    a(Ins("Lodd_last:", "label"))
    ops += iteration(1, 1, True, False, True, "oZ", sequential)
    ops += drain(1)
    if DUMP == "O":
        ops += dump_and_exit([("a", i) for i in range(128)] +
                             [("v", V_M), ("v", V_M + 1), ("v", V_L), ("v", V_L + 1)], inp)
    ops += epilogue()
    a(Ins("Lrow_done:", "label"))
    return ops


# ----------------------------------------------------------------------------------------------
# hazard check: distances (in issued instructions, s_nop n counting n + 1) that the hardware does
# not enforce by itself on gfx950.  Conservative figures; the schedule is built to respect them,
# this pass only proves it.
# ----------------------------------------------------------------------------------------------
MFMA_RESULT_TO_OTHER = 18       # MFMA writes regs -> non-MFMA touches them / MFMA reads them as A or B
VALU_TO_MFMA = 4                # VALU writes regs -> MFMA reads them
TRANS_TO_USE = 2                # transcendental result -> its use
VALU_SGPR_TO_VALU = 3           # VALU writes an SGPR (or vcc) -> a VALU reads it (2 on gfx950)
LANE_OP_TO_USE = 2              # permlane swap / readfirstlane result -> its use
VALU_TO_LANE_OP = 2             # VALU writes a VGPR -> readfirstlane / permlane swap reads it (1 / 2 on gfx950)


def check_hazards(ops, first_only=False):
    """Returns [(index in ops, missing wait states, instruction, reason)]; with first_only the
    first violation as [(index, missing)]."""
    pos = 0
    last_mfma_wr = {}
    last_valu_wr = {}
    last_trans_wr = {}
    last_lane_wr = {}
    problems = []
    for idx, ins in enumerate(ops):
        if ins.kind in ("label", "barrier", "wait"):
            # a label is reached by fall-through or by a jump from a place that is at least as far
            # from the producers (every jump here follows a barrier or leaves a loop body's end)
            pos += 1
            continue
        if ins.kind == "nop":
            pos += int(ins.text.split()[1]) + 1
            continue
        need, why = 0, ""

        def rule(last, r, dist, what):
            nonlocal need, why
            if r in last and dist - (pos - last[r]) > need:
                need, why = dist - (pos - last[r]), f"{r} written by {what} {pos - last[r]} back"

        for r in ins.rd | ins.wr:
            same_acc_chain = ins.kind == "mfma" and r in ins.wr and r in ins.rd
            if not same_acc_chain:
                rule(last_mfma_wr, r, MFMA_RESULT_TO_OTHER, "MFMA")
        for r in ins.rd:
            if ins.kind == "mfma":
                rule(last_valu_wr, r, VALU_TO_MFMA, "VALU")
            if ins.kind == "lane" and r[0] == "v":
                rule(last_valu_wr, r, VALU_TO_LANE_OP, "VALU")
            if ins.kind in ("valu", "trans", "lane") and r[0] == "s":
                rule(last_valu_wr, r, VALU_SGPR_TO_VALU, "VALU")
            if ins.kind in ("valu", "trans", "mfma", "vmem", "lds"):
                rule(last_lane_wr, r, LANE_OP_TO_USE, "a lane operation")
            rule(last_trans_wr, r, TRANS_TO_USE, "a transcendental")
        if need > 0:
            if first_only:
                return [(idx, need)]
            problems.append((idx, need, ins.text, why))
        for r in ins.wr:
            if ins.kind == "mfma":
                last_mfma_wr[r] = pos
            else:
                last_mfma_wr.pop(r, None)
                if ins.kind in ("valu", "trans", "lane"):
                    last_valu_wr[r] = pos
                if ins.kind == "trans":
                    last_trans_wr[r] = pos
                else:
                    last_trans_wr.pop(r, None)
                if ins.kind == "lane":
                    last_lane_wr[r] = pos
                else:
                    last_lane_wr.pop(r, None)
        pos += 1
    return problems


def skipped_view(ops):
    """Indices of `ops` on the path that takes every forward conditional branch (the rare blocks:
    causal mask, rescale, copy guards, lse): distances across a skipped block are the short ones."""
    keep = []
    skip_to = None
    for i, ins in enumerate(ops):
        if skip_to is not None:
            if ins.kind == "label" and ins.text == skip_to + ":":
                skip_to = None
            continue
        keep.append(i)
        if ins.kind == "salu" and ins.text.startswith("s_cbranch_"):
            target = ins.text.split()[1]
            later = any(o.kind == "label" and o.text == target + ":" for o in ops[i + 1:i + 1200])
            if later and target.startswith(("Lnomask", "Lnoresc", "Lnok", "Lnolse", "Lnopull")):
                skip_to = target
    return keep


def all_hazards(ops, first_only=False):
    """Hazards on the path through every rare block and on the path round all of them."""
    found = check_hazards(ops, first_only)
    if found and first_only:
        return found
    view = skipped_view(ops)
    sub = check_hazards([ops[i] for i in view], first_only)
    mapped = [(view[p[0]],) + tuple(p[1:]) for p in sub]
    return (found + mapped) if not first_only else mapped


def fix_hazards(ops):
    """Inserts s_nop where the order of `ops` would violate a rule of check_hazards."""
    out = list(ops)
    for _ in range(400):
        problems = all_hazards(out, first_only=True)
        if not problems:
            return out
        idx, need = problems[0]
        while need > 0:
            k = min(need, 8)
            out.insert(idx, nop(k - 1))
            need -= k
    raise SystemExit("fix_hazards did not converge")


INP = {}          # operand names of the inline-asm inputs, filled by emit()


INPUTS = ["t", "q", "o", "lse", "k", "vt", "col", "n", "u", "causal", "lds", "kbytes", "vbytes", "c0", "cnt"]


def emit(path, sequential=False):
    inp = {name: f"%{i + 1}" for i, name in enumerate(INPUTS)}      # %0 is the output operand
    INP.update(inp)
    ops = fix_hazards(row_program(inp, sequential))
    # the queue position pulled for the next row (valid in lane 0 of wave 0)
    ops.append(valu(f"v_mov_b32 %0, v{V_T + 28}", vr(V_T + 28), ()))
    problems = all_hazards(ops)
    if problems:
        for p in problems[:20]:
            print("hazard:", p, file=sys.stderr)
        raise SystemExit(f"{len(problems)} hazard(s) in the generated schedule")
    clob_v = [f"v{i}" for i in range(32, 256)]
    clob_a = [f"a{i}" for i in range(0, 256)]
    clob_s = [f"s{i}" for i in range(40, 96)]
    with open(path, "w") as f:
        f.write("// generated by gen_attn_w64.py -- do not edit\n")
        f.write("asm volatile(\n")
        for ins in ops:
            f.write(f'    "{ins.text}\\n\\t"\n')
        f.write('    : "=&v"(pulled_next)\n')
        f.write('    : "v"(t), "s"(q_row), "s"(o_row), "s"(lse_row), "s"(k_head), "s"(vt_head), "s"(col_row),\n')
        f.write('      "s"(n_entries), "s"(u), "s"(causal), "s"(lds_base), "s"(k_bytes), "s"(vt_bytes), "s"(c_first),\n')
        f.write('      "s"(pull_counter)\n')
        clob = ", ".join(f'"{c}"' for c in clob_v + clob_a + clob_s + ["vcc", "scc", "memory"])
        f.write(f"    : {clob});\n")
    n_mfma = sum(1 for i in ops if i.kind == "mfma")
    print(f"{path}: {len(ops)} instructions, {n_mfma} MFMAs", file=sys.stderr)


if __name__ == "__main__":
    out = sys.argv[1] if len(sys.argv) > 1 else os.path.join(os.path.dirname(os.path.abspath(__file__)),
                                                              "prism_attn_w64_body.inc")
    emit(out, sequential="--sequential" in sys.argv)
