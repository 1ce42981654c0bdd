#!/usr/bin/env python3
"""Writes qsv_gate_asm.h: the text of the inline-assembly gate interpreter of the fused pass
kernel (gfx950).  Run by build.py before hipcc; the header is also committed so that the source
tree compiles as it stands.

Why assembly: the 32 amplitude registers of a lane must stay where they are across the whole
operation list.  A C++ switch over operation kinds makes the compiler copy all of them at every
merge point; one asm block with tied operands and its own scalar dispatch does not.

The block executes consecutive gate operations (2x2 unitary on a register bit, CNOT with the
control in a register bit, CNOT with the control elsewhere in the index) and returns at the first
operation of any other kind, leaving the operation pointer on it.

Fixed scalar registers (declared as clobbers): s[80:81] operation word, s82 kind, s83 field a,
s[84:85] scratch / saved exec, s[86:87] matrix address, s[88:95] matrix, s[96:97] operation
pointer.  Operation word: x = kind | a<<8 | b<<16 | c<<24, y = arg.
"""
import os

R = 4
NR = 1 << R
OP_U, OP_CX_REG, OP_CX_DYN = 3, 4, 5


def u_pair(a, b):
    """(r_a,i_a) has the target bit 0, (r_b,i_b) has it 1; matrix m0..m7 = s88..s95 =
    (m00r, m00i, m01r, m01i, m10r, m10i, m11r, m11i).  Four interleaved chains; the last step of
    each overwrites an input that is dead by then."""
    ra, ia, rb, ib = "%%[r%d]" % a, "%%[i%d]" % a, "%%[r%d]" % b, "%%[i%d]" % b
    t = ["%[t0]", "%[t1]", "%[t2]", "%[t3]"]
    return [
        "v_mul_f32 %s, s88, %s" % (t[0], ra),
        "v_mul_f32 %s, s89, %s" % (t[1], ra),
        "v_mul_f32 %s, s92, %s" % (t[2], ra),
        "v_mul_f32 %s, s93, %s" % (t[3], ra),
        "v_fma_f32 %s, -s89, %s, %s" % (t[0], ia, t[0]),
        "v_fma_f32 %s, s88, %s, %s" % (t[1], ia, t[1]),
        "v_fma_f32 %s, -s93, %s, %s" % (t[2], ia, t[2]),
        "v_fma_f32 %s, s92, %s, %s" % (t[3], ia, t[3]),
        "v_fma_f32 %s, s90, %s, %s" % (t[0], rb, t[0]),
        "v_fma_f32 %s, s91, %s, %s" % (t[1], rb, t[1]),
        "v_fma_f32 %s, s94, %s, %s" % (t[2], rb, t[2]),
        "v_fma_f32 %s, s95, %s, %s" % (t[3], rb, t[3]),
        "v_fma_f32 %s, -s91, %s, %s" % (ra, ib, t[0]),
        "v_fma_f32 %s, s90, %s, %s" % (ia, ib, t[1]),
        "v_fma_f32 %s, -s95, %s, %s" % (rb, ib, t[2]),
        "v_fma_f32 %s, s94, %s, %s" % (ib, ib, t[3]),
    ]


def swap_pair(a, b):
    return ["v_swap_b32 %%[r%d], %%[r%d]" % (a, b), "v_swap_b32 %%[i%d], %%[i%d]" % (a, b)]


def gen():
    L = []
    emit = L.append
    lab = lambda name: "L_%s_%%=" % name

    emit("s_mov_b32 s96, %[opslo]")
    emit("s_mov_b32 s97, %[opshi]")
    emit(lab("fetch") + ":")
    emit("s_load_dwordx2 s[80:81], s[96:97], 0x0")
    emit("s_waitcnt lgkmcnt(0)")
    emit("s_and_b32 s82, s80, 0xff")
    emit("s_bfe_u32 s83, s80, 0x80008")
    emit("s_cmp_eq_u32 s82, %d" % OP_U)
    emit("s_cbranch_scc1 " + lab("u"))
    emit("s_cmp_eq_u32 s82, %d" % OP_CX_REG)
    emit("s_cbranch_scc1 " + lab("cxr"))
    emit("s_cmp_eq_u32 s82, %d" % OP_CX_DYN)
    emit("s_cbranch_scc1 " + lab("cxd"))
    emit("s_branch " + lab("exit"))

    # ---- 2x2 unitary on register bit a; matrix = (arg == ovr_id) ? *ovr : mbase[arg]
    emit(lab("u") + ":")
    emit("s_bfe_u32 s84, s80, 0x80010")          # b: matrix depends on the state row
    emit("s_and_b32 s84, s84, %[nonuni]")        # ... and rows differ per lane: not ours
    emit("s_cmp_lg_u32 s84, 0")
    emit("s_cbranch_scc1 " + lab("exit"))
    emit("s_cmp_eq_u32 s81, %[ovrid]")
    emit("s_cbranch_scc1 " + lab("uovr"))
    emit("s_lshl_b32 s84, s81, 5")
    emit("s_mov_b32 s86, %[mlo]")
    emit("s_mov_b32 s87, %[mhi]")
    emit("s_add_u32 s86, s86, s84")
    emit("s_addc_u32 s87, s87, 0")
    emit("s_branch " + lab("uld"))
    emit(lab("uovr") + ":")
    emit("s_mov_b32 s86, %[olo]")
    emit("s_mov_b32 s87, %[ohi]")
    emit(lab("uld") + ":")
    emit("s_load_dwordx8 s[88:95], s[86:87], 0x0")
    emit("s_waitcnt lgkmcnt(0)")
    for j in range(R - 1):
        emit("s_cmp_eq_u32 s83, %d" % j)
        emit("s_cbranch_scc1 " + lab("u%d" % j))
    for j in reversed(range(R)):
        emit(lab("u%d" % j) + ":")
        for i in range(NR):
            if i & (1 << j):
                continue
            L.extend(u_pair(i, i | (1 << j)))
        emit("s_branch " + lab("next"))

    # ---- CNOT, control = register bit b, target = register bit a
    emit(lab("cxr") + ":")
    emit("s_bfe_u32 s84, s80, 0x80010")
    emit("s_lshl_b32 s85, s83, 2")
    emit("s_add_u32 s84, s84, s85")
    combos = [(jt, jc) for jt in range(R) for jc in range(R) if jt != jc]
    for jt, jc in combos:
        emit("s_cmp_eq_u32 s84, %d" % (jt * 4 + jc))
        emit("s_cbranch_scc1 " + lab("x%d%d" % (jt, jc)))
    emit("s_branch " + lab("next"))               # unknown combination: no-op (never planned)
    for jt, jc in combos:
        emit(lab("x%d%d" % (jt, jc)) + ":")
        for i in range(NR):
            if (i & (1 << jc)) and not (i & (1 << jt)):
                L.extend(swap_pair(i, i | (1 << jt)))
        emit("s_branch " + lab("next"))

    # ---- CNOT, control = index bit b outside the register run (lane-dependent), target = a
    emit(lab("cxd") + ":")
    emit("s_bfe_u32 s86, s80, 0x80010")
    emit("s_lshl_b64 s[84:85], 1, s86")
    emit("v_and_b32 %[tc], s84, %[e0lo]")
    emit("v_and_b32 %[t0], s85, %[e0hi]")
    emit("v_or_b32 %[tc], %[tc], %[t0]")
    emit("v_cmp_ne_u32 vcc, 0, %[tc]")
    emit("s_and_saveexec_b64 s[84:85], vcc")
    emit("s_cbranch_execz " + lab("cxdone"))
    for j in range(R - 1):
        emit("s_cmp_eq_u32 s83, %d" % j)
        emit("s_cbranch_scc1 " + lab("d%d" % j))
    for j in reversed(range(R)):
        emit(lab("d%d" % j) + ":")
        for i in range(NR):
            if not (i & (1 << j)):
                L.extend(swap_pair(i, i | (1 << j)))
        if j != 0:
            emit("s_branch " + lab("cxdone"))
    emit(lab("cxdone") + ":")
    emit("s_mov_b64 exec, s[84:85]")

    emit(lab("next") + ":")
    emit("s_add_u32 s96, s96, 8")
    emit("s_addc_u32 s97, s97, 0")
    emit("s_branch " + lab("fetch"))
    emit(lab("exit") + ":")
    emit("s_mov_b32 %[opslo], s96")
    emit("s_mov_b32 %[opshi], s97")
    return L


def render():
    lines = gen()
    out = ["// Generated by gen_gate_asm.py -- do not edit by hand.",
           "// Inline-assembly gate interpreter of the fused pass kernel; see the generator for the",
           "// register map and the reason it is assembly.",
           "#pragma once",
           "#define QSV_GATE_LOOP_ASM \\"]
    for ln in lines:
        out.append('    "%s\\n\\t" \\' % ln)
    out.append('    ""')
    regs = ", ".join('"s%d"' % i for i in range(80, 98))
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
