"""The C-ABI library loads and exports every symbol declared in include/qsv.h (no GPU needed),
and argument errors are reported before anything touches a device."""
import ctypes
import os
import re

from paper_2602_13140_amd import binding as qb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "qsv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qsv_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    L = qb.load()
    names = declared_symbols()
    assert {"qsv_create", "qsv_amp_encode", "qsv_apply_layers", "qsv_measure",
            "qsv_param_shift_grad"} <= set(names)
    for name in names:
        assert hasattr(L, name), name


def test_binding_struct_layouts_match_header():
    assert ctypes.sizeof(qb.qsv_circuit) == 7 * 4
    assert ctypes.sizeof(qb.qsv_measure_req) == 64
    assert ctypes.sizeof(qb.qsv_loss) == 24 and qb.qsv_loss.targets_dev.offset == 16
    assert qb.qsv_measure_req.out_dev.offset == 56


def test_create_rejects_bad_arguments_without_a_gpu():
    L = qb.load()
    h = ctypes.c_void_p()
    fake = ctypes.c_void_p(0x1000)
    big = qb.qsv_workspace_bytes(4, 2)
    assert L.qsv_create(None, 4, 2, 0, None, fake, fake, big) == qb.QSV_ERR_INVALID_ARG
    assert L.qsv_create(ctypes.byref(h), 0, 2, 0, None, fake, fake, big) == qb.QSV_ERR_INVALID_ARG
    assert L.qsv_create(ctypes.byref(h), 31, 2, 0, None, fake, fake, big) == qb.QSV_ERR_INVALID_ARG
    assert L.qsv_create(ctypes.byref(h), 4, 0, 0, None, fake, fake, big) == qb.QSV_ERR_INVALID_ARG
    assert L.qsv_create(ctypes.byref(h), 4, 2, 0, None, None, fake, big) == qb.QSV_ERR_INVALID_ARG
    assert L.qsv_create(ctypes.byref(h), 4, 2, 0, None, ctypes.c_void_p(0x1004), fake, big) == qb.QSV_ERR_INVALID_ARG
    assert L.qsv_create(ctypes.byref(h), 4, 2, 0, None, fake, fake, 16) == qb.QSV_ERR_WORKSPACE
    assert b"workspace" in L.qsv_last_error(None)
    assert h.value is None


def test_workspace_size_grows_with_the_state():
    assert qb.qsv_workspace_bytes(26, 1) > qb.qsv_workspace_bytes(20, 1) > 0
    assert qb.qsv_workspace_bytes(10, 1024) > qb.qsv_workspace_bytes(10, 1)
    c = qb.make_circuit(10, [2, 3], 2)
    extra = qb.qsv_grad_workspace_bytes(16, 256, c) - qb.qsv_workspace_bytes(16, 256)
    assert 256 * 11 * (8 << 16) <= extra <= 256 * 11 * (8 << 16) + 4096
    assert qb.qsv_grad_workspace_bytes(16, 256, qb.make_circuit(1, [9], 1)) == 0
