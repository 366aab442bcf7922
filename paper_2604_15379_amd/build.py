"""Build the HIP library for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_PKG, "csrc")
LIB_PATH = os.path.join(_PKG, "libfleet.so")
SOURCES = [os.path.join(_CSRC, "fleet.hip"), os.path.join(_CSRC, "graph.cpp")]
_DEPS = SOURCES + [os.path.join(_CSRC, "kernels.hip.inc"), os.path.join(_CSRC, "graph.hpp"),
                   os.path.join(_PKG, "..", "include", "fleet.h")]


def hipcc_command(out: str = LIB_PATH, extra=()) -> list:
    return ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
            # packed-FP32 instructions are not to be generated on the test machines
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wno-unused-value", *extra, "-o", out, *SOURCES]


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile libfleet.so in-tree.  With force=False an up-to-date library is kept."""
    if not force and os.path.exists(LIB_PATH) and \
            all(os.path.getmtime(LIB_PATH) >= os.path.getmtime(d) for d in _DEPS):
        return LIB_PATH
    cmd = hipcc_command()
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    if verbose:
        print(res.stderr)
    return LIB_PATH
