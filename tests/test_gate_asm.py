"""Host-logic checks of the generated gate-interpreter assembly (no GPU): the control flow must
not fall from one operation's code into another's, every label must exist exactly once, and the
committed header must be what the generator writes."""
import os
import re

from paper_2602_13140_amd.csrc import gen_gate_asm as g

INTENDED_FALLTHROUGH = {"L_top", "L_uhave", "L_unopf", "L_u3", "L_d3", "L_cxdone", "L_xphave", "L_xpw",
                        "L_xpr", "L_zm3", "L_zdone"}


def test_no_unintended_fall_through():
    lines = g.gen()
    for i, ln in enumerate(lines):
        if ln.endswith(":") and i > 0:
            prev = lines[i - 1]
            if prev.startswith("s_branch") or prev.endswith(":"):
                continue
            name = ln[:-1].replace("_%=", "")
            assert name in INTENDED_FALLTHROUGH, (name, prev)


def test_labels_defined_once_and_targets_exist():
    lines = g.gen()
    labels = [ln[:-1] for ln in lines if ln.endswith(":")]
    assert len(labels) == len(set(labels))
    for ln in lines:
        m = re.match(r"s_c?branch\w*\s+(L_\w+_%=)$", ln)
        if m:
            assert m.group(1) in labels, ln


def test_exit_is_reached_only_with_nothing_in_flight():
    """Every jump to the exit comes from the dispatch right after the wait at the top, or from the
    unitary's early test, which sits before any load of that operation is issued."""
    lines = g.gen()
    top = lines.index("L_top_%=:")
    assert lines[top + 1] == "s_waitcnt lgkmcnt(0)"
    for i, ln in enumerate(lines):
        if "L_exit_%=" in ln and not ln.endswith(":"):
            seg = lines[top:i]
            assert not any(x.startswith(("s_load", "ds_read", "ds_write")) for x in seg[2:]), ln


def test_only_fixed_scalar_registers_in_the_clobber_range_are_used():
    text = "\n".join(g.gen())
    for m in re.finditer(r"\bs\[?(\d+)", text):
        assert g.FIRST_SGPR <= int(m.group(1)) <= g.LAST_SGPR, m.group(0)


def test_committed_header_is_current():
    path = os.path.join(os.path.dirname(os.path.abspath(g.__file__)), "qsv_gate_asm.h")
    assert open(path).read() == g.render()
