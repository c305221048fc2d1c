"""Build libtbn.so (HIP, gfx950 only) next to this file with hipcc.

Usage: ``python -m paper_2407_12075_amd.build``.  The library is built in-tree so that it travels
with the source tree; nothing is installed.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libtbn.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# The compiler the hand-scheduled kernels were validated with.  Several kernels read LDS through inline assembly
# and hand the destination registers to the compiler before the data has arrived; that is sound only if the
# compiler puts nothing that touches them between a read and its wait.  asm_check.py verifies this on the
# generated assembly; with another compiler version the check (and the GPU tests) have to be repeated before
# these strings are changed.
VALIDATED_HIP_VERSION = "7.2.26015"
VALIDATED_CLANG = "roc-7.2.0 26014"
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the fully unrolled MFMA chains of the convolution kernel are longer than the default limit of
    # `#pragma unroll`; partly unrolled, their register arrays would go to scratch memory
    "-mllvm", "-pragma-unroll-threshold=100000",
    "-Wall", "-Wno-unused-function",
]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    cmd = [HIPCC, *FLAGS, "-c", src, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(_compile, srcs))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", *objs, "-o", LIB]
    subprocess.run(cmd, check=True)
    if verbose:
        print(f"built {LIB} from {len(srcs)} sources")
    return LIB


def hipcc_version() -> str:
    return subprocess.run([HIPCC, "--version"], capture_output=True, text=True, check=True).stdout


if __name__ == "__main__":
    build()
