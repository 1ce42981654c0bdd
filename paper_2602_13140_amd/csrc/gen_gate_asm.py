#!/usr/bin/env python3
"""Writes qsv_gate_asm.h: the text of the inline-assembly gate interpreter of the fused pass
kernel (gfx950).  Run by build.py before hipcc; the header is also committed so that the source
tree compiles as it stands.

Why assembly: the 32 amplitude registers of a lane must stay where they are across the whole
operation list.  A C++ switch over operation kinds makes the compiler copy all of them at every
merge point; one asm block with tied operands and its own scalar dispatch does not.  It also
lets the next operation word and the next matrix be fetched while the current gate computes.

The block executes consecutive operations (2x2 unitary on a register bit, CNOT with the control
in a register bit, CNOT with the control elsewhere in the index or given by the parity of several
index bits, the three forms of CZ sign flips,
and the transpose through LDS that moves the register run) and returns at the first operation of any other kind, leaving the
operation pointer on it and no scalar load or LDS access in flight.

LDS layout: one plane of 2^T floats through which the real parts go first and then the imaginary
parts (the default), or two planes for both at once.  Element tau of a plane sits at index
tau ^ ((tau >> 4) & 31): the XOR spreads every layout's 32 consecutive lanes over the 32 banks,
costs no space, and, XOR being linear, the address of register element k is (lane's part) ^ off(k)
with off(k) the XOR of the offsets of k's set bits.  A layout is therefore described by four
offsets (those of elements 1, 2, 4, 8), kept in vector registers, and the elements are visited in
Gray-code order, so that each address is the previous one XOR one of the four: one vector-only
v_xor per element (a vector instruction with a scalar operand issues at 4.2 cycles per wavefront
on this chip, one with vector operands only at 2.5).
The dynamic LDS segment starts at byte 0 (the kernel has no static LDS), so no base is added.

Operation word: x = kind | a<<8 | b<<16 | c<<24, y = arg.  For a unitary, arg is the index of its
matrix in execution order, so consecutive unitaries read consecutive 32-byte matrices and the
next one can be prefetched (the table is padded by one entry for the last prefetch).

Fixed scalar registers (declared as clobbers; the text below names them s52..s56 and s68..s99,
_renumbered() packs them into s36..s72, which leaves the compiler enough of the 96 scalar registers
the kernel is limited to (eight wavefronts per SIMD) to do without spills):
  s[52:55] landing place of a layout's four offsets on their way to vector registers
  s68 layout whose offsets sit in %[ba0..3] (-1: none, the compiler may have used them since)
  s69 one-plane transposes: the exchange crosses wavefronts
  s56 index (in execution order) of the matrix in s[72:79], -1: none; s[70:71] its address
  s[72:79] matrix of the stream: the one in use until its vector copies are made, then the next
  s[80:81] current operation word     s82 kind   s83 field a
  s[84:85] scratch / saved exec       s[86:87] scratch address
  s[88:95] shifted matrix of a gradient row
  s[96:97] operation pointer          s[98:99] next operation word
"""
import os
import re

R = 4
NR = 1 << R
OP_XPOSE, OP_U, OP_CX_REG, OP_CX_DYN, OP_CZ_REG, OP_CZ_MIX, OP_CZ_LANE, OP_CX_CHAIN, OP_CX_PAR, OP_CX_LANE = 2, 3, 4, 5, 6, 7, 8, 9, 10, 12
# the chains of CNOTs between neighbouring register bits, numbered as in the planner:
# (direction, control of the first, count); direction 0: controls go up, 1: down
CX_CHAINS = [(0, 0, 3), (1, 2, 3), (0, 0, 2), (0, 1, 2), (1, 2, 2), (1, 1, 2)]
FIRST_SGPR, LAST_SGPR = 36, 72      # after _renumbered()
GRAY = [i ^ (i >> 1) for i in range(NR)]        # element visited at step i
GRAY_BIT = [0] + [(i & -i).bit_length() - 1 for i in range(1, NR)]   # bit that changes on entering step i


def u_pair(a, b, variant="g"):
    """(r_a,i_a) has the target bit 0, (r_b,i_b) has it 1; matrix m0..m7 = vector copies of
    s88..s95 = (m00r, m00i, m01r, m01i, m10r, m10i, m11r, m11i): a vector instruction with a scalar
    operand issues at 4.2 cycles per wavefront on this chip, one with vector operands only at 2.5.
    Four interleaved chains; the last step of each overwrites an input that is dead by then.
    Variants leave out the products with
    imaginary parts that are stored as exact zeros: "g" none (16 instructions), "a" m00i (14),
    "r" m00i and m01i (first row real, 12), "c" m00i and m10i (first column real, 12)."""
    ra, ia, rb, ib = "%%[r%d]" % a, "%%[i%d]" % a, "%%[r%d]" % b, "%%[i%d]" % b
    t = ["%[t0]", "%[t1]", "%[t2]", "%[t3]"]
    mul = lambda d, m, x: "v_mul_f32 %s, %s, %s" % (d, m, x)
    fma = lambda d, m, x, acc: "v_fma_f32 %s, %s, %s, %s" % (d, m, x, acc)
    if variant == "g":
        return [
            mul(t[0], "%[m0]", ra), mul(t[1], "%[m1]", ra), mul(t[2], "%[m4]", ra), mul(t[3], "%[m5]", ra),
            fma(t[0], "-%[m1]", ia, t[0]), fma(t[1], "%[m0]", ia, t[1]),
            fma(t[2], "-%[m5]", ia, t[2]), fma(t[3], "%[m4]", ia, t[3]),
            fma(t[0], "%[m2]", rb, t[0]), fma(t[1], "%[m3]", rb, t[1]),
            fma(t[2], "%[m6]", rb, t[2]), fma(t[3], "%[m7]", rb, t[3]),
            fma(ra, "-%[m3]", ib, t[0]), fma(ia, "%[m2]", ib, t[1]),
            fma(rb, "-%[m7]", ib, t[2]), fma(ib, "%[m6]", ib, t[3]),
        ]
    if variant == "a":
        return [
            mul(t[0], "%[m0]", ra), mul(t[1], "%[m0]", ia), mul(t[2], "%[m4]", ra), mul(t[3], "%[m5]", ra),
            fma(t[2], "-%[m5]", ia, t[2]), fma(t[3], "%[m4]", ia, t[3]),
            fma(t[0], "%[m2]", rb, t[0]), fma(t[1], "%[m3]", rb, t[1]),
            fma(t[2], "%[m6]", rb, t[2]), fma(t[3], "%[m7]", rb, t[3]),
            fma(ra, "-%[m3]", ib, t[0]), fma(ia, "%[m2]", ib, t[1]),
            fma(rb, "-%[m7]", ib, t[2]), fma(ib, "%[m6]", ib, t[3]),
        ]
    if variant == "r":
        return [
            mul(t[0], "%[m0]", ra), mul(t[1], "%[m0]", ia), mul(t[2], "%[m4]", ra), mul(t[3], "%[m5]", ra),
            fma(t[2], "-%[m5]", ia, t[2]), fma(t[3], "%[m4]", ia, t[3]),
            fma(t[2], "%[m6]", rb, t[2]), fma(t[3], "%[m7]", rb, t[3]),
            fma(ra, "%[m2]", rb, t[0]), fma(ia, "%[m2]", ib, t[1]),
            fma(rb, "-%[m7]", ib, t[2]), fma(ib, "%[m6]", ib, t[3]),
        ]
    assert variant == "c"
    return [
        mul(t[0], "%[m0]", ra), mul(t[1], "%[m0]", ia), mul(t[2], "%[m4]", ra), mul(t[3], "%[m4]", ia),
        fma(t[0], "%[m2]", rb, t[0]), fma(t[1], "%[m3]", rb, t[1]),
        fma(t[2], "%[m6]", rb, t[2]), fma(t[3], "%[m7]", rb, t[3]),
        fma(ra, "-%[m3]", ib, t[0]), fma(ia, "%[m2]", ib, t[1]),
        fma(rb, "-%[m7]", ib, t[2]), fma(ib, "%[m6]", ib, t[3]),
    ]


CHAIN_FORM = "move"     # "swap": every cycle by v_swap_b32


def chain_swaps(direction, first, count):
    """The chain's CNOTs (control c, target c + 1) as one permutation of the 16 register elements.  A cycle of
    k elements takes k - 1 swaps (v_swap_b32, 8.2 cycles each) or k + 1 moves through a temporary (2.5
    cycles each): cycles of two are swapped, longer ones moved.  Measured on one box, alternating the two
    builds: moves take 0.8 % off the 26-qubit and 20-qubit configurations now that their passes are
    heavy (when the passes were lighter and waited for memory the same change cost 0.6 %)."""
    src = list(range(NR))                  # src[i]: which old element ends up in place i
    for k in range(count):
        c = first + k if direction == 0 else first - k
        t = c + 1
        for i in range(NR):
            if (i >> c) & 1 and not (i >> t) & 1:
                j = i | (1 << t)
                src[i], src[j] = src[j], src[i]
    out, seen = [], [False] * NR
    for s0 in range(NR):
        if seen[s0] or src[s0] == s0:
            continue
        cyc, cur = [], s0
        while not seen[cur]:
            seen[cur] = True
            cyc.append(cur)
            cur = src[cur]
        if CHAIN_FORM == "move" and len(cyc) > 2:
            # place cyc[k] receives the old content of cyc[k+1]; the first one's goes round through a temporary
            for part, tmp in (("r", "%[t0]"), ("i", "%[t1]")):
                reg = lambda k: "%%[%s%d]" % (part, k)
                out.append("v_mov_b32 %s, %s" % (tmp, reg(cyc[0])))
                for a, b in zip(cyc, cyc[1:]):
                    out.append("v_mov_b32 %s, %s" % (reg(a), reg(b)))
                out.append("v_mov_b32 %s, %s" % (reg(cyc[-1]), tmp))
            continue
        # place cyc[k] must receive the old content of cyc[k+1]: swap neighbours along the cycle
        for a, b in zip(cyc, cyc[1:]):
            out.extend(swap_pair(a, b))
    return out


def swap_pair(a, b):
    return ["v_swap_b32 %%[r%d], %%[r%d]" % (a, b), "v_swap_b32 %%[i%d], %%[i%d]" % (a, b)]


def gen(planes=2, perlane=False):
    """perlane: the variant for kernels whose tiles hold several state rows, where a unitary whose
    matrix depends on the row is left to the caller."""
    assert planes in (1, 2)
    L = []
    emit = L.append
    lab = lambda name: "L_%s_%%=" % name
    ALIGN = ".p2align 6"                          # branch targets start an instruction-fetch line

    def prefetch_next_word():
        emit("s_load_dwordx2 s[98:99], s[96:97], 0x8")

    emit("s_mov_b32 s96, %[opslo]")
    emit("s_mov_b32 s97, %[opshi]")
    emit("s_mov_b32 s56, -1")                     # no matrix prefetched yet
    emit("s_mov_b32 s68, -1")
    emit("s_load_dwordx2 s[98:99], s[96:97], 0x0")
    emit("s_branch " + lab("top"))
    emit(ALIGN)
    emit(lab("next") + ":")                       # falls through to the top: one jump per operation
    emit("s_add_u32 s96, s96, 8")
    emit("s_addc_u32 s97, s97, 0")
    emit(lab("top") + ":")
    emit("s_waitcnt lgkmcnt(0)")                  # next word and prefetched matrix have landed
    emit("s_mov_b64 s[80:81], s[98:99]")
    emit("s_and_b32 s82, s80, 0xff")
    emit("s_bfe_u32 s83, s80, 0x80008")
    emit("s_cmp_eq_u32 s82, %d" % OP_U)
    emit("s_cbranch_scc1 " + lab("u"))
    emit("s_cmp_eq_u32 s82, %d" % OP_CX_CHAIN)
    emit("s_cbranch_scc1 " + lab("cxc"))
    emit("s_cmp_eq_u32 s82, %d" % OP_CX_REG)
    emit("s_cbranch_scc1 " + lab("cxr"))
    emit("s_cmp_eq_u32 s82, %d" % OP_CX_DYN)
    emit("s_cbranch_scc1 " + lab("cxd"))
    emit("s_cmp_eq_u32 s82, %d" % OP_XPOSE)
    emit("s_cbranch_scc1 " + lab("xp"))
    emit("s_cmp_eq_u32 s82, %d" % OP_CX_LANE)
    emit("s_cbranch_scc1 " + lab("cxl"))
    emit("s_cmp_eq_u32 s82, %d" % OP_CX_PAR)
    emit("s_cbranch_scc1 " + lab("cxp"))
    emit("s_cmp_eq_u32 s82, %d" % OP_CZ_REG)
    emit("s_cbranch_scc1 " + lab("zr"))
    emit("s_cmp_eq_u32 s82, %d" % OP_CZ_MIX)
    emit("s_cbranch_scc1 " + lab("zm"))
    emit("s_cmp_eq_u32 s82, %d" % OP_CZ_LANE)
    emit("s_cbranch_scc1 " + lab("zl"))
    emit("s_branch " + lab("exit"))

    # ---- 2x2 unitary on register bit a; matrix = (arg == ovrid) ? *ovr : mbase[arg].
    # s[72:79] holds the matrix of the stream with index s56 (-1: none), s[70:71] its address; the
    # multiply sequences read vector copies, so the buffer is free for the next matrix of the stream
    # as soon as the copies are made.  Every scalar instruction here competes with the vector ones
    # for issue slots, hence the short common path: two compares, the variant and bit dispatch.
    emit(ALIGN)
    emit(lab("u") + ":")
    if perlane:
        emit("s_bfe_u32 s84, s80, 0x80010")      # b: matrix depends on the state row
        emit("s_and_b32 s84, s84, %[nonuni]")    # ... and rows differ per lane: not ours
        emit("s_cmp_lg_u32 s84, 0")
        emit("s_cbranch_scc1 " + lab("exit"))
    emit("s_cmp_eq_u32 s81, %[ovrid]")
    emit("s_cbranch_scc1 " + lab("uovr"))
    emit("s_cmp_eq_u32 s81, s56")
    emit("s_cbranch_scc0 " + lab("uld"))
    emit(lab("uhave") + ":")
    # pick the multiply sequence from the zeros the matrix builder stored
    emit("s_cmp_lg_u32 s73, 0")
    emit("s_cbranch_scc1 " + lab("ug"))
    emit("s_cmp_eq_u32 s75, 0")
    emit("s_cbranch_scc1 " + lab("ur"))
    emit("s_cmp_eq_u32 s77, 0")
    emit("s_cbranch_scc1 " + lab("uc"))
    for variant in "argc":
        emit(ALIGN)
        emit(lab("u" + variant) + ":")
        # the multiply sequences read vector registers only: stage the entries this variant uses
        used = sorted({int(m) for ln in u_pair(0, 1, variant) for m in re.findall(r"%\[m(\d)\]", ln)})
        for k in used:
            emit("v_mov_b32 %%[m%d], s%d" % (k, 72 + k))
        emit("s_add_u32 s70, s70, 32")            # prefetch the next matrix of the stream
        emit("s_addc_u32 s71, s71, 0")
        emit("s_add_u32 s56, s56, 1")
        emit("s_load_dwordx8 s[72:79], s[70:71], 0x0")
        if variant == "g":
            emit(lab("ugj") + ":")                # the shifted matrix of a gradient row joins here
        prefetch_next_word()
        for j in range(R - 1):
            emit("s_cmp_eq_u32 s83, %d" % j)
            emit("s_cbranch_scc1 " + lab("u%s%d" % (variant, j)))
        for j in reversed(range(R)):
            emit(ALIGN)
            emit(lab("u%s%d" % (variant, j)) + ":")
            for i in range(NR):
                if i & (1 << j):
                    continue
                L.extend(u_pair(i, i | (1 << j), variant))
            emit("s_branch " + lab("next"))
    # not the prefetched one (first unitary of a tile, or the one after a shifted matrix): fetch it
    emit(lab("uld") + ":")
    emit("s_lshl_b32 s84, s81, 5")
    emit("s_add_u32 s70, %[mlo], s84")
    emit("s_addc_u32 s71, %[mhi], 0")
    emit("s_mov_b32 s56, s81")
    emit("s_load_dwordx8 s[72:79], s[70:71], 0x0")
    emit("s_waitcnt lgkmcnt(0)")
    emit("s_branch " + lab("uhave"))
    # the shifted matrix of a gradient row: not part of the stream, general multiply sequence
    emit(lab("uovr") + ":")
    emit("s_mov_b32 s86, %[olo]")
    emit("s_mov_b32 s87, %[ohi]")
    emit("s_load_dwordx8 s[88:95], s[86:87], 0x0")
    emit("s_waitcnt lgkmcnt(0)")
    for k in range(8):
        emit("v_mov_b32 %%[m%d], s%d" % (k, 88 + k))
    emit("s_branch " + lab("ugj"))

    # ---- CNOT, control = register bit b, target = register bit a
    emit(ALIGN)
    emit(lab("cxr") + ":")
    prefetch_next_word()
    emit("s_bfe_u32 s84, s80, 0x80010")
    emit("s_lshl_b32 s85, s83, 2")
    emit("s_add_u32 s84, s84, s85")
    # searched in this order: first the neighbours a CNOT ring produces (target just above the
    # control), since every compare is an instruction that competes with the vector ones for issue
    combos = [(jc + 1, jc) for jc in range(R - 1)]
    combos += [(jt, jc) for jt in range(R) for jc in range(R) if jt != jc and (jt, jc) not in combos]
    for jt, jc in combos:
        emit("s_cmp_eq_u32 s84, %d" % (jt * 4 + jc))
        emit("s_cbranch_scc1 " + lab("x%d%d" % (jt, jc)))
    emit("s_branch " + lab("next"))               # unknown combination: no-op (never planned)
    for jt, jc in combos:
        emit(ALIGN)
        emit(lab("x%d%d" % (jt, jc)) + ":")
        for i in range(NR):
            if (i & (1 << jc)) and not (i & (1 << jt)):
                L.extend(swap_pair(i, i | (1 << jt)))
        emit("s_branch " + lab("next"))

    # ---- chain of CNOTs between neighbouring register bits: arg numbers the chain
    emit(ALIGN)
    emit(lab("cxc") + ":")
    prefetch_next_word()
    for k in range(len(CX_CHAINS) - 1):
        emit("s_cmp_eq_u32 s81, %d" % k)
        emit("s_cbranch_scc1 " + lab("c%d" % k))
    for k in reversed(range(len(CX_CHAINS))):
        emit(ALIGN)
        emit(lab("c%d" % k) + ":")
        L.extend(chain_swaps(*CX_CHAINS[k]))
        emit("s_branch " + lab("next"))

    # ---- CNOT, control = index bit b outside the register run (lane-dependent), target = a
    emit(ALIGN)
    emit(lab("cxd") + ":")
    prefetch_next_word()
    emit("s_bfe_u32 s86, s80, 0x80010")
    emit("s_lshl_b64 s[84:85], 1, s86")
    emit("v_and_b32 %[tc], s84, %[e0lo]")
    emit("v_and_b32 %[t0], s85, %[e0hi]")
    emit("v_or_b32 %[tc], %[tc], %[t0]")
    emit("v_cmp_ne_u32 vcc, 0, %[tc]")
    emit(lab("cxdx") + ":")
    emit("s_and_saveexec_b64 s[84:85], vcc")
    emit("s_cbranch_execz " + lab("cxdone"))
    for j in range(R - 1):
        emit("s_cmp_eq_u32 s83, %d" % j)
        emit("s_cbranch_scc1 " + lab("d%d" % j))
    for j in reversed(range(R)):
        emit(ALIGN)
        emit(lab("d%d" % j) + ":")
        for i in range(NR):
            if not (i & (1 << j)):
                L.extend(swap_pair(i, i | (1 << j)))
        if j != 0:
            emit("s_branch " + lab("cxdone"))
    emit(lab("cxdone") + ":")
    emit("s_mov_b64 exec, s[84:85]")
    emit("s_branch " + lab("next"))

    # ---- CNOT, target = register bit a, control = parity of the lane's index bits in arg (a mask
    # over the low 32 bits of the extended index, none of them in the register run): the condition,
    # then the swaps of the handler above
    emit(ALIGN)
    emit(lab("cxp") + ":")
    prefetch_next_word()
    emit("v_and_b32 %[tc], s81, %[e0lo]")
    emit("v_bcnt_u32_b32 %[tc], %[tc], 0")
    emit("v_and_b32 %[tc], 1, %[tc]")
    emit("v_cmp_ne_u32 vcc, 0, %[tc]")
    emit("s_branch " + lab("cxdx"))



    # ---- CNOT, control = register bit a, target = bit b of the lane number: every lane trades its
    # eight amplitudes with the control set for the partner lane's (lane ^ 2^b).  b = 0, 1: DPP
    # quad permutes, in place; b >= 2: ds_bpermute_b32 (lane crossbar of the LDS unit, no memory
    # involved) with the partner's byte address in %[tc].
    emit(ALIGN)
    emit(lab("cxl") + ":")
    prefetch_next_word()
    emit("s_bfe_u32 s84, s80, 0x80010")           # b
    emit("s_cmp_eq_u32 s84, 0")
    emit("s_cbranch_scc1 " + lab("cxlq0"))
    emit("s_cmp_eq_u32 s84, 1")
    emit("s_cbranch_scc1 " + lab("cxlq1"))
    emit("s_lshl_b32 s85, 1, s84")
    emit("v_xor_b32 %[tc], s85, %[thr]")
    emit("v_and_b32 %[tc], 63, %[tc]")
    emit("v_lshlrev_b32 %[tc], 2, %[tc]")
    for j in range(R - 1):
        emit("s_cmp_eq_u32 s83, %d" % j)
        emit("s_cbranch_scc1 " + lab("cxlb%d" % j))
    for j in reversed(range(R)):
        emit(ALIGN)
        emit(lab("cxlb%d" % j) + ":")
        for k in range(NR):
            if (k >> j) & 1:
                emit("ds_bpermute_b32 %%[r%d], %%[tc], %%[r%d]" % (k, k))
                emit("ds_bpermute_b32 %%[i%d], %%[tc], %%[i%d]" % (k, k))
        emit("s_branch " + lab("next"))           # the wait at the top covers the exchange
    for b, perm in ((0, "[1,0,3,2]"), (1, "[2,3,0,1]")):
        emit(lab("cxlq%d" % b) + ":")
        for j in range(R - 1):
            emit("s_cmp_eq_u32 s83, %d" % j)
            emit("s_cbranch_scc1 " + lab("cxlq%d_%d" % (b, j)))
        for j in reversed(range(R)):
            emit(ALIGN)
            emit(lab("cxlq%d_%d" % (b, j)) + ":")
            for k in range(NR):
                if (k >> j) & 1:
                    for part in "ri":
                        emit("v_mov_b32_dpp %%[%s%d], %%[%s%d] quad_perm:%s row_mask:0xf bank_mask:0xf"
                             % (part, k, part, k, perm))
            emit("s_branch " + lab("next"))

    def flip(part, k):
        return "v_xor_b32 %%[%s%d], 0x80000000, %%[%s%d]" % (part, k, part, k)

    # ---- CZ between register bits a < b: the amplitudes with both bits set change sign
    emit(ALIGN)
    emit(lab("zr") + ":")
    prefetch_next_word()
    emit("s_bfe_u32 s84, s80, 0x80010")
    emit("s_lshl_b32 s85, s83, 2")
    emit("s_add_u32 s84, s84, s85")
    pairs = [(ja, jb) for ja in range(R) for jb in range(ja + 1, R)]
    for ja, jb in pairs:
        emit("s_cmp_eq_u32 s84, %d" % (ja * 4 + jb))
        emit("s_cbranch_scc1 " + lab("zr%d%d" % (ja, jb)))
    emit("s_branch " + lab("next"))               # unknown combination: no-op (never planned)
    for ja, jb in pairs:
        emit(lab("zr%d%d" % (ja, jb)) + ":")
        for k in range(NR):
            if (k >> ja) & 1 and (k >> jb) & 1:
                emit(flip("r", k))
                emit(flip("i", k))
        emit("s_branch " + lab("next"))

    # ---- CZ between register bit a and index bit b outside the run: lanes whose bit b is set
    # flip the sign of the amplitudes with register bit a set
    emit(ALIGN)
    emit(lab("zm") + ":")
    prefetch_next_word()
    emit("s_bfe_u32 s86, s80, 0x80010")
    emit("s_lshl_b64 s[84:85], 1, s86")
    emit("v_and_b32 %[tc], s84, %[e0lo]")
    emit("v_and_b32 %[t0], s85, %[e0hi]")
    emit("v_or_b32 %[tc], %[tc], %[t0]")
    emit("v_cmp_ne_u32 vcc, 0, %[tc]")
    emit("s_and_saveexec_b64 s[84:85], vcc")
    emit("s_cbranch_execz " + lab("zdone"))
    for j in range(R - 1):
        emit("s_cmp_eq_u32 s83, %d" % j)
        emit("s_cbranch_scc1 " + lab("zm%d" % j))
    for j in reversed(range(R)):
        emit(lab("zm%d" % j) + ":")
        for k in range(NR):
            if (k >> j) & 1:
                emit(flip("r", k))
                emit(flip("i", k))
        emit("s_branch " + lab("zdone"))

    # ---- CZ rungs (mask in arg, bit q = rung (q, q+1)) between index bits outside the run: one
    # sign per lane, parity of popcount(e0 & (e0 >> 1) & mask); the mask lies below bit 31
    emit(ALIGN)
    emit(lab("zl") + ":")
    prefetch_next_word()
    emit("v_lshrrev_b32 %[t0], 1, %[e0lo]")
    emit("v_and_b32 %[t0], %[t0], %[e0lo]")
    emit("v_and_b32 %[t0], s81, %[t0]")
    emit("v_bcnt_u32_b32 %[t0], %[t0], 0")
    emit("v_and_b32 %[t0], 1, %[t0]")
    emit("v_cmp_ne_u32 vcc, 0, %[t0]")
    emit("s_and_saveexec_b64 s[84:85], vcc")
    emit("s_cbranch_execz " + lab("zdone"))
    for k in range(NR):
        emit(flip("r", k))
        emit(flip("i", k))
    emit(lab("zdone") + ":")
    emit("s_mov_b64 exec, s[84:85]")
    emit("s_branch " + lab("next"))

    # ---- transpose: move the register run from layout scur to layout a (field a of the word).
    # The four address offsets of a layout come from a 4-dword table row (one scalar load) and go to
    # vector registers: %[ba0..3] for the layout named in s68 (-1: none), %[bb0..3] for the layout
    # being moved to.
    def load_offsets(sreg):
        emit("s_lshl_b32 s84, %s, 4" % sreg)
        emit("s_add_u32 s86, %[tablo], s84")
        emit("s_addc_u32 s87, %[tabhi], 0")
        emit("s_load_dwordx4 s[52:55], s[86:87], 0x0")

    def offsets_to(prefix):
        for j in range(4):
            emit("v_mov_b32 %%[%s%d], s%d" % (prefix, j, 52 + j))

    tmps = ["%[t0]", "%[t1]", "%[t2]", "%[t3]"]

    def walk(base, prefix, access):
        """Visits the 16 register elements in Gray-code order; access(k, address register)."""
        prev = base
        for i in range(NR):
            if i:
                t = tmps[i % 4]
                emit("v_xor_b32 %s, %s, %%[%s%d]" % (t, prev, prefix, GRAY_BIT[i]))
                prev = t
            access(GRAY[i], prev)

    def lane_part(dst):
        """dst = byte address part of the lane in layout scur; also refreshes e0."""
        # tau = ((thr >> s) << (s + 4)) | (thr & ((1 << s) - 1))
        emit("v_lshrrev_b32 %[t0], %[scur], %[thr]")
        emit("s_add_u32 s84, %[scur], 4")
        emit("v_lshlrev_b32 %[t0], s84, %[t0]")
        emit("s_lshl_b32 s85, 1, %[scur]")
        emit("s_sub_u32 s85, s85, 1")
        emit("v_and_b32 %[t1], s85, %[thr]")
        emit("v_or_b32 %[t0], %[t0], %[t1]")          # t0 = tau of the lane (register bits zero)
        emit("v_lshrrev_b32 %[t1], 4, %[t0]")
        emit("v_and_b32 %[t1], 31, %[t1]")
        emit("v_xor_b32 %[t1], %[t1], %[t0]")
        emit("v_lshlrev_b32 " + dst + ", 2, %[t1]")   # swz(tau) * 4
        # extended index of the lane: e0 = tile_base | (tau & cmask) | ((tau >> c) << w), w < 32
        emit("v_lshrrev_b32 %[t1], %[c], %[t0]")
        emit("v_and_b32 %[t2], %[cmask], %[t0]")
        emit("v_lshlrev_b32 %[t3], %[w], %[t1]")
        emit("v_or_b32 %[t2], %[t2], %[t3]")
        emit("v_or_b32 %[e0lo], %[tblo], %[t2]")
        emit("s_sub_u32 s84, 32, %[w]")
        emit("v_lshrrev_b32 %[t1], s84, %[t1]")
        emit("v_or_b32 %[e0hi], %[tbhi], %[t1]")

    emit(ALIGN)
    emit(lab("xp") + ":")
    prefetch_next_word()
    emit("s_cmp_eq_u32 s68, %[scur]")
    emit("s_cbranch_scc1 " + lab("xphave"))
    load_offsets("%[scur]")
    emit("s_waitcnt lgkmcnt(0)")
    offsets_to("ba")
    emit(lab("xphave") + ":")
    emit("s_bfe_u32 s84, s80, 0x80018")           # c: barrier before the writes
    emit("s_cmp_eq_u32 s84, 0")
    emit("s_cbranch_scc1 " + lab("xpw"))
    emit("s_barrier")
    emit(lab("xpw") + ":")
    if planes == 2:
        walk("%[ldsb]", "ba", lambda k, t: emit(
            "ds_write2st64_b32 %s, %%[r%d], %%[i%d] offset1:%%[pl64]" % (t, k, k)))
        # new layout: its offsets first (they arrive while the lane's own part is computed)
        emit("s_mov_b32 %[scur], s83")
        load_offsets("%[scur]")
        lane_part("%[ldsb]")
        emit("s_waitcnt lgkmcnt(0)")              # own writes are in LDS, new offsets are here
        offsets_to("ba")
        emit("s_mov_b32 s68, %[scur]")
        emit("s_bfe_u32 s84, s80, 0x80010")       # b: the exchange crosses wavefronts
        emit("s_cmp_eq_u32 s84, 0")
        emit("s_cbranch_scc1 " + lab("xpr"))
        emit("s_barrier")
        emit(lab("xpr") + ":")

        def read2(k, t):
            emit("ds_read_b32 %%[r%d], %s" % (k, t))
            emit("ds_read_b32 %%[i%d], %s offset:%%[plane4]" % (k, t))
        walk("%[ldsb]", "ba", read2)
        emit("s_branch " + lab("next"))           # the wait at the top covers the reads
    else:
        # One plane: real parts go through it first, then the imaginary parts.  The offsets of the
        # new layout sit in %[bb0..3] until the end, the lane's new address part in ldsn.  A
        # wavefront's LDS operations execute in order, so the steps need a wait and a barrier
        # between them only when the exchange crosses wavefronts (flag b, kept in s69).
        def sync(name):
            emit("s_cmp_eq_u32 s69, 0")
            emit("s_cbranch_scc1 " + lab(name))
            emit("s_waitcnt lgkmcnt(0)")
            emit("s_barrier")
            emit(lab(name) + ":")

        def writes(part):
            walk("%[ldsb]", "ba", lambda k, t: emit("ds_write_b32 %s, %%[%s%d]" % (t, part, k)))

        def reads(part):
            walk("%[ldsn]", "bb", lambda k, t: emit("ds_read_b32 %%[%s%d], %s" % (part, k, t)))

        emit("s_bfe_u32 s69, s80, 0x80010")
        writes("r")
        emit("s_mov_b32 %[scur], s83")
        load_offsets("%[scur]")
        lane_part("%[ldsn]")
        emit("s_waitcnt lgkmcnt(0)")              # new offsets are here (and own writes landed)
        offsets_to("bb")
        emit("s_cmp_eq_u32 s69, 0")
        emit("s_cbranch_scc1 " + lab("xpr"))
        emit("s_barrier")
        emit(lab("xpr") + ":")
        reads("r")
        sync("xpw2")
        writes("i")
        sync("xpr2")
        reads("i")
        for j in range(4):                        # the new layout's offsets become the current ones
            emit("v_mov_b32 %%[ba%d], %%[bb%d]" % (j, j))
        emit("s_mov_b32 s68, %[scur]")
        emit("v_mov_b32 %[ldsb], %[ldsn]")
        emit("s_branch " + lab("next"))           # the wait at the top covers the reads

    emit(lab("exit") + ":")                       # reached right after the wait: nothing in flight
    emit("s_mov_b32 %[opslo], s96")
    emit("s_mov_b32 %[opshi], s97")
    return [_renumbered(ln) for ln in L]


def _renumbered(line):
    """Packs the block's scalar registers: s52..s55 -> s36..s39, s68..s99 -> s40..s71 (both shifts
    keep the alignment that register pairs, quads and octets need), s56 -> s72."""
    import re

    def new(n):
        n = int(n)
        if 52 <= n <= 55:
            return n - 16
        if n == 56:
            return 72
        assert 68 <= n <= 99, n
        return n - 28
    line = re.sub(r"\bs\[(\d+):(\d+)\]", lambda m: "s[%d:%d]" % (new(m.group(1)), new(m.group(2))), line)
    return re.sub(r"\bs(\d+)\b", lambda m: "s%d" % new(m.group(1)), line)


def render():
    out = ["// Generated by gen_gate_asm.py -- do not edit by hand.",
           "// Inline-assembly gate interpreter of the fused pass kernel; see the generator for the",
           "// register map and the reason it is assembly.  _2P: transposes through two LDS planes",
           "// (real, imaginary) at once; _1P: through one plane, real parts first.  _ROWS: for tiles that",
           "// hold several state rows (returns at a unitary whose matrix depends on the row).",
           "#pragma once"]
    for planes in (2, 1):
        for perlane in (False, True):
            out.append("#define QSV_GATE_LOOP_ASM_%dP%s \\" % (planes, "_ROWS" if perlane else ""))
            for ln in gen(planes, perlane):
                out.append('    "%s\\n\\t" \\' % ln)
            out.append('    ""')
    regs = ", ".join('"s%d"' % i for i in range(FIRST_SGPR, LAST_SGPR + 1))
    out.append("#define QSV_GATE_LOOP_CLOBBERS %s, \"vcc\", \"scc\", \"memory\"" % regs)
    return "\n".join(out) + "\n"


def write(path=None):
    path = path or os.path.join(os.path.dirname(os.path.abspath(__file__)), "qsv_gate_asm.h")
    text = render()
    if not os.path.exists(path) or open(path).read() != text:
        with open(path, "w") as f:
            f.write(text)
    return path


if __name__ == "__main__":
    print(write())
