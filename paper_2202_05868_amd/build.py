"""Build the C-ABI library (host C++ + HIP kernels for gfx950) in-tree with hipcc.

    python -m paper_2202_05868_amd.build

produces ``paper_2202_05868_amd/libvbr_spmm.so`` next to this file.  The library is a plain
shared object behind ``include/vbr_spmm.h``; it does not link against PyTorch.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libvbr_spmm.so")
SOURCES = ["sa1_reorder.cpp", "vbr_build.cpp", "vbr_spmm.hip", "csr_spmm.hip", "denominators.hip"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = False) -> str:
    """Compile every source for gfx950 and link the shared library.  Always recompiles."""
    cmd = [hipcc(), "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
           # packed fp32 instructions are kept out of the generated device code
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-mpopcnt", "-pthread",
           "-Wall", "-Wno-unused-command-line-argument",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    for s in SOURCES:
        p = os.path.join(CSRC, s)
        cmd += (["-x", "hip", p] if s.endswith(".hip") else ["-x", "c++", p])
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd += ["-o", tmp]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(ln for ln in res.stdout.splitlines() if "packed-fp32-ops" not in ln)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
