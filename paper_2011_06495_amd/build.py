"""Builds the C-ABI library (libmv.so) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libmv.so")
SOURCES = [os.path.join(CSRC, "mv_api.hip"), os.path.join(CSRC, "mv_codec.hip"),
           os.path.join(CSRC, "mv_quant.hip")]
HEADERS = [os.path.join(CSRC, h) for h in ("mv_kernels.hpp", "mv_common.hpp", "mv_stream.hpp", "mv_select.hpp",
                                               "mv_mask.hpp", "mv_add_drop.hpp", "mv_random_select.hpp")] + [
           os.path.join(os.path.dirname(_HERE), "include", "mv.h")]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # the aggregate is a plain sum then one multiply: never contract into FMAs
    "-ffp-contract=off",
    # keep fp32 denormals (a denormal magnitude still orders above zero)
    "-fno-gpu-flush-denormals-to-zero",
    # scalar fp32 ALU ops only: no packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def needs_build() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(s) > t for s in SOURCES + HEADERS)


def build_lib(force: bool = True, verbose: bool = False) -> str:
    """Compiles libmv.so.  With force=False an up-to-date library is kept."""
    if not force and not needs_build():
        return LIB_PATH
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB_PATH + ".tmp.%d" % os.getpid()
    cmd = [hipcc, *HIPCC_FLAGS, *SOURCES, "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build_lib(verbose=True))
