"""Builds the shared libraries in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(HERE, "libcascade_moe.so")
SYNTH_LIB = os.path.join(HERE, "libmoe_synth.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 VALU forms are switched off on purpose (scalar fp32 code only)
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("build failed: " + " ".join(cmd) + "\n" + r.stdout + r.stderr)
    return r


def _check_no_scratch(stderr: str) -> None:
    """Refuse a build in which any kernel spills registers to scratch memory: the expert kernels are
    sized to stay in registers, and a spilling variant of them has been seen to give wrong results."""
    name = None
    for line in stderr.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split("[")[0].strip()
        elif "ScratchSize [bytes/lane]:" in line:
            size = int(line.split("ScratchSize [bytes/lane]:")[1].split("[")[0].strip())
            if size != 0:
                raise RuntimeError(f"kernel {name} uses {size} bytes/lane of scratch (register spill)")


def _check_mfma_readers(tmp: str) -> None:
    """Refuse a build whose generated code reads a matrix-core result sooner than the hardware delivers it on some
    path (see mfma_hazard_check.py): the device assembly the compiler left in `tmp` is scanned."""
    from . import mfma_hazard_check
    asm = [f for f in os.listdir(tmp) if f.endswith(".s") and "gfx950" in f]
    if len(asm) != 1:
        raise RuntimeError(f"expected one gfx950 assembly file in {tmp}, found {asm}")
    bad = mfma_hazard_check.check(open(os.path.join(tmp, asm[0])).read())
    if bad:
        lines = [f"  {k}: v_mfma #{i} read after {slots} issue slots by `{what}`" for k, i, what, slots in bad[:10]]
        raise RuntimeError(f"{len(bad)} too-early reader(s) of a matrix-core result in the generated code:\n" + "\n".join(lines))


def build_all(verbose: bool = False) -> None:
    import shutil
    import tempfile
    obj_c = os.path.join(HERE, "cascade_ctrl.o")
    tmp = tempfile.mkdtemp(prefix="moe_build_")
    try:
        obj_k = os.path.join(tmp, "moe_kernels.o")
        r = _run([HIPCC] + HIP_FLAGS + ["-Rpass-analysis=kernel-resource-usage", "-save-temps=obj", "-I", INCLUDE, "-c",
                                       os.path.join(CSRC, "moe_kernels.hip"), "-o", obj_k])
        _check_no_scratch(r.stderr)
        _check_mfma_readers(tmp)
        _build_rest(obj_k, obj_c, verbose)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)


def _build_rest(obj_k: str, obj_c: str, verbose: bool) -> None:
    # host policy code: plain C++ with contraction off so decisions replay identically everywhere
    _run(["g++", "-O2", "-std=c++17", "-fPIC", "-ffp-contract=off", "-I", INCLUDE, "-c",
          os.path.join(CSRC, "cascade_ctrl.cpp"), "-o", obj_c])
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", obj_k, obj_c, "-o", LIB])
    _run([HIPCC] + HIP_FLAGS + ["-shared", os.path.join(CSRC, "synth_fill.hip"), "-o", SYNTH_LIB])
    os.remove(obj_c)
    if verbose:
        print("built", LIB, SYNTH_LIB)


if __name__ == "__main__":
    build_all(verbose=True)
