"""Compile the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libpmpd.so")
SOURCES = [os.path.join(CSRC, "pmpd_host.cpp"), os.path.join(CSRC, "pmpd_gemv.hip"), os.path.join(CSRC, "pmpd_prefill.hip"),
           os.path.join(CSRC, "pmpd_fp16.hip"), os.path.join(CSRC, "pmpd_learned.hip"),
           os.path.join(CSRC, "pmpd_skinny.hip"), os.path.join(CSRC, "pmpd_block16.hip")]
HEADERS = [os.path.join(CSRC, "pmpd_common.hpp"), os.path.join(CSRC, "pmpd_device.hpp"), os.path.join(CSRC, "pmpd_sumword.hpp"), os.path.join(CSRC, "pmpd_prefill_deal.hpp"), os.path.join(ROOT, "include", "pmpd.h")]

# packed-fp32 VALU forms are switched off for all device code of this library.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def build(verbose: bool = False, extra_flags=()) -> str:
    """Always recompiles; returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-o", LIB, *SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout)
        raise RuntimeError("hipcc failed building libpmpd.so")
    return LIB


def up_to_date() -> bool:
    if not os.path.exists(LIB):
        return False
    t = os.path.getmtime(LIB)
    return all(os.path.getmtime(p) <= t for p in SOURCES + HEADERS)


if __name__ == "__main__":
    print(build(verbose=True))
