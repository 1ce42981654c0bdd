"""Host-logic checks of the generated gate-interpreter assembly (no GPU): the control flow must
not fall from one operation's code into another's, every label must exist exactly once, and the
committed header must be what the generator writes."""
import os
import re

from paper_2602_13140_amd.csrc import gen_gate_asm as g

INTENDED_FALLTHROUGH = {"L_top", "L_uhave", "L_ugj", "L_ua", "L_ua3", "L_ur3", "L_ug3", "L_uc3",
                        "L_d3", "L_c5", "L_cxdone", "L_cxdx", "L_cxlb3", "L_cxlq0_3", "L_cxlq1_3", "L_xphave", "L_xpw", "L_xpr", "L_xpw2", "L_xpr2", "L_zm3", "L_zdone"}


import pytest

PLANES = pytest.mark.parametrize("planes", [1, 2, -1, -2])      # negative: the several-rows-per-tile variant


def gen(planes):
    return g.gen(abs(planes), planes < 0)


def code_lines(planes):
    """The generated instructions and labels, without assembler directives (alignment)."""
    return [ln for ln in gen(planes) if not ln.startswith(".")]


@PLANES
def test_no_unintended_fall_through(planes):
    lines = code_lines(planes)
    for i, ln in enumerate(lines):
        if ln.endswith(":") and i > 0:
            prev = lines[i - 1]
            if prev.startswith("s_branch") or prev.endswith(":"):
                continue
            name = ln[:-1].replace("_%=", "")
            assert name in INTENDED_FALLTHROUGH, (name, prev)


@PLANES
def test_labels_defined_once_and_targets_exist(planes):
    lines = code_lines(planes)
    labels = [ln[:-1] for ln in lines if ln.endswith(":")]
    assert len(labels) == len(set(labels))
    for ln in lines:
        m = re.match(r"s_c?branch\w*\s+(L_\w+_%=)$", ln)
        if m:
            assert m.group(1) in labels, ln


@PLANES
def test_exit_is_reached_only_with_nothing_in_flight(planes):
    """Every jump to the exit comes from the dispatch right after the wait at the top, or from the
    unitary's early test, which sits before any load of that operation is issued."""
    lines = code_lines(planes)
    top = lines.index("L_top_%=:")
    assert lines[top + 1] == "s_waitcnt lgkmcnt(0)"
    for i, ln in enumerate(lines):
        if "L_exit_%=" in ln and not ln.endswith(":"):
            seg = lines[top:i]
            assert not any(x.startswith(("s_load", "ds_read", "ds_write")) for x in seg[2:]), ln


@PLANES
def test_only_fixed_scalar_registers_in_the_clobber_range_are_used(planes):
    text = "\n".join(code_lines(planes))
    for m in re.finditer(r"\bs\[?(\d+)", text):
        assert g.FIRST_SGPR <= int(m.group(1)) <= g.LAST_SGPR, m.group(0)


def test_committed_header_is_current():
    path = os.path.join(os.path.dirname(os.path.abspath(g.__file__)), "qsv_gate_asm.h")
    assert open(path).read() == g.render()


def _run_valu(lines, regs, sregs):
    """Executes v_mul_f32 / v_fma_f32 lines (matrix entry as first operand, optional negation) on floats."""
    val = lambda tok: -sregs[tok[1:]] if tok.startswith("-") else sregs[tok]
    for ln in lines:
        op, rest = ln.split(" ", 1)
        a = [x.strip() for x in rest.split(",")]
        if op == "v_mul_f32":
            regs[a[0]] = val(a[1]) * regs[a[2]]
        else:
            assert op == "v_fma_f32"
            regs[a[0]] = val(a[1]) * regs[a[2]] + regs[a[3]]


def test_unitary_multiply_sequences_compute_the_matrix_product():
    """Each variant of the 2x2 update equals the complex matrix-vector product when the imaginary
    parts it leaves out are zero, and the variants have 16/14/12/12 instructions."""
    import numpy as np
    g0 = np.random.Generator(np.random.PCG64(5))
    zero = {"g": [], "a": [1], "r": [1, 3], "c": [1, 5]}        # indices into m00r..m11i
    size = {"g": 16, "a": 14, "r": 12, "c": 12}
    for variant in "garc":
        m = g0.standard_normal(8)
        m[zero[variant]] = 0.0
        sregs = {"%%[m%d]" % k: m[k] for k in range(8)}
        a = g0.standard_normal(2) + 1j * g0.standard_normal(2)
        regs = {"%[r2]": a[0].real, "%[i2]": a[0].imag, "%[r6]": a[1].real, "%[i6]": a[1].imag}
        lines = g.u_pair(2, 6, variant)
        assert len(lines) == size[variant]
        _run_valu(lines, regs, sregs)
        mat = (m[0::2] + 1j * m[1::2]).reshape(2, 2)
        want = mat @ a
        got = np.array([regs["%[r2]"] + 1j * regs["%[i2]"], regs["%[r6]"] + 1j * regs["%[i6]"]])
        assert np.allclose(got, want, atol=1e-13), variant


def test_gray_walk_visits_every_element_at_its_swizzled_offset():
    """The transposes reach register element GRAY[i] by XORing one of four per-layout offsets onto the
    previous address; the result must be the element's own offset swz(k << s) * 4 in every layout."""
    swz = lambda x: x ^ ((x >> 4) & 31)
    assert sorted(g.GRAY) == list(range(16))
    for s in range(12):
        basis = [swz((1 << j) << s) * 4 for j in range(4)]
        addr = 0
        for i in range(16):
            if i:
                addr ^= basis[g.GRAY_BIT[i]]
            assert addr == swz(g.GRAY[i] << s) * 4, (s, i)


@pytest.mark.parametrize("planes", [1, 2])
def test_transposes_use_vector_operands_only(planes):
    """Address arithmetic of the transposes: every v_xor takes vector registers only (a scalar operand
    would cost 4.2 instead of 2.5 cycles per wavefront), and every element is written and read."""
    lines = code_lines(planes)
    xors = [ln for ln in lines if ln.startswith("v_xor_b32 %[t") and "%[b" in ln]
    assert xors and all(re.fullmatch(r"v_xor_b32 %\[t\d\], %\[(t\d|ldsb|ldsn)\], %\[b[ab]\d\]", ln) for ln in xors)
    for part, count in (("r", 1), ("i", 1)):
        for k in range(16):
            reads = [ln for ln in lines if ln.startswith("ds_read_b32 %%[%s%d]," % (part, k))]
            assert len(reads) == count, (part, k)


@PLANES
def test_branch_targets_reached_by_jumps_are_aligned(planes):
    """Where the code of the operations sits relative to the instruction-fetch lines changed the run
    time of the whole kernel by 5 to 9 % between two otherwise equal builds; the handlers' entry
    points are therefore aligned to 64 bytes."""
    lines = gen(planes)
    for name in ("L_next_%=:", "L_u_%=:", "L_cxr_%=:", "L_cxd_%=:", "L_xp_%=:", "L_ug3_%=:", "L_x10_%=:"):
        assert lines[lines.index(name) - 1] == ".p2align 6", name


def test_row_dependent_exit_only_in_the_variant_for_several_rows_per_tile():
    for planes in (1, 2):
        assert not any("%[nonuni]" in ln for ln in g.gen(planes, False))
        assert any("%[nonuni]" in ln for ln in g.gen(planes, True))


def test_chain_swaps_equal_the_cnots_one_after_the_other():
    """Every chain's sequence of swaps and moves, run on 16 distinct values, gives what its CNOTs give in
    turn, in about as many instructions as the CNOTs one by one would take."""
    for direction, first, count in g.CX_CHAINS:
        regs = {}
        for k in range(16):
            regs["%%[r%d]" % k] = 100 + k
            regs["%%[i%d]" % k] = 200 + k
        lines = g.chain_swaps(direction, first, count)
        assert len(lines) <= 16 * count + 8
        for ln in lines:
            op, rest = ln.split(" ", 1)
            x, y = [t.strip() for t in rest.split(",")]
            if op == "v_swap_b32":
                regs[x], regs[y] = regs[y], regs[x]
            else:
                assert op == "v_mov_b32" and (x in regs or x in ("%[t0]", "%[t1]"))
                regs[x] = regs[y]
        want = list(range(16))
        for k in range(count):
            c = first + k if direction == 0 else first - k
            t = c + 1
            assert 0 <= c and t < 4
            for i in range(16):
                if (i >> c) & 1 and not (i >> t) & 1:
                    j = i | (1 << t)
                    want[i], want[j] = want[j], want[i]
        assert [regs["%%[r%d]" % k] - 100 for k in range(16)] == want, (direction, first, count)
        assert [regs["%%[i%d]" % k] - 200 for k in range(16)] == want
