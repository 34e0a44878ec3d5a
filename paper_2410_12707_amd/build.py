"""Builds libadatopk.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree, and next to it
libadatopk_measure.so: the same sources compiled with ADATOPK_MEASURE_BUILD, which adds the
benchmark-only hooks of include/adatopk_measure.h (per-kernel dispatch timing, plain streaming
kernels).  The product library carries none of them."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libadatopk.so")
MEASURE_LIB = os.path.join(HERE, "libadatopk_measure.so")
SOURCES = [os.path.join(CSRC, "adatopk.hip"), os.path.join(CSRC, "adatopk_host.cpp")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra",
    # packed-fp32 instruction forms are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def build_library(verbose: bool = False, out: str = LIB, defines=()) -> str:
    """Compiles the library to `out`; `defines` are extra -D macros (launch-shape overrides)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-D" + d for d in defines] + ["-o", out] + SOURCES
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return out


def build_measure_library(verbose: bool = False) -> str:
    return build_library(verbose, MEASURE_LIB, ("ADATOPK_MEASURE_BUILD",))


def library_is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = SOURCES + [os.path.join(ROOT, "include", "adatopk.h"), os.path.join(ROOT, "include", "adatopk_measure.h"),
                      os.path.join(CSRC, "wire_layout.h")]
    return any(os.path.getmtime(d) > t for d in deps)


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_measure_library(verbose=True))
