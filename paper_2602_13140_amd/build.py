"""Builds libqsv.so (hand-written HIP for gfx950 + host planner + C ABI) in-tree with hipcc."""
import os
import subprocess
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libqsv.so")
SOURCES = ["qsv_api.cpp", "qsv_plan.cpp", "qsv_kernels.hip"]
HEADERS = ["qsv_plan.h", "qsv_kernels.h", "gen_gate_asm.py", os.path.join(ROOT, "include", "qsv.h")]


def hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def needs_build():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    files = [os.path.join(CSRC, s) for s in SOURCES]
    files += [h if os.path.isabs(h) else os.path.join(CSRC, h) for h in HEADERS]
    return any(os.path.getmtime(f) > t for f in files)


def build(force=True, verbose=False):
    """Compile for gfx950.  Packed-FP32 instruction selection is switched off on purpose."""
    if not force and not needs_build():
        return LIB
    from paper_2602_13140_amd.csrc import gen_gate_asm  # noqa: E402  (regenerate the asm header)
    gen_gate_asm.write()
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-x", "hip",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    cmd += ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build(force=True, verbose=True)
    print(LIB)
