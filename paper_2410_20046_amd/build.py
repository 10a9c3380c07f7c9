"""Builds libdqrm.so (the gfx950 HIP kernels + C ABI) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libdqrm.so")
SOURCES = [os.path.join(CSRC, "dqrm_api.hip")]
HEADERS = [os.path.join(CSRC, f) for f in ("dqrm_device.hpp", "dqrm_fwd.hpp", "dqrm_bwd.hpp", "dqrm_update.hpp",
                                             "dqrm_merge.hpp", "dqrm_dense.hpp")] + [
    os.path.join(ROOT, "include", "dqrm.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # results are compared bit for bit with a CPU oracle: one rounding per
    # operation, correctly rounded fp32 division
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt",
    # do not let the compiler form packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    m = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > m for f in SOURCES + HEADERS)


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compile the library.  Cross-compiles for gfx950; needs no GPU."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", LIB] + SOURCES
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + r.stdout)
    return LIB


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
