"""Builds libcolbandit.so (HIP kernels + C-ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcolbandit.so")
SOURCES = ["cb_api.hip", "cb_kernels.hip", "cb_dense.hip", "cb_quant.hip", "cb_baselines.hip"]
HEADERS = ["cb_device.h", "cb_launch.h", os.path.join("..", "..", "include", "colbandit.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-Xarch_device", "-fno-honor-nans", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed fp32 VALU forms are kept off for the device code of this library
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build_library(force: bool = False, verbose: bool = False) -> str:
    if not force and not _stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                                            text=True)))
        objs.append(obj)
    for cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
        if verbose and out.strip():
            print(out, file=sys.stderr)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    return LIB


ABI_CHECK_SRC = os.path.join(HERE, "..", "tests", "native", "abi_check.cpp")
ABI_CHECK = os.path.join(HERE, "..", "tests", "native", "abi_check.bin")


def build_abi_check() -> str:
    """Compiles tests/native/abi_check.cpp, a plain C++ host program that drives the C-ABI
    without Python, against the built library (found at run time through its rpath)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-x", "hip", ABI_CHECK_SRC,
           "-x", "none", "-L" + HERE, "-lcolbandit",
           "-Wl,-rpath,$ORIGIN/../../paper_2602_02827_amd", "-o", ABI_CHECK]
    subprocess.run(cmd, check=True)
    return ABI_CHECK


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
