"""Build the HIP library for gfx950 with hipcc (cross-compiles without a GPU).

The persistent kernel exists in seven flavours (one translation unit each, see
csrc/kernel_variant.hip); the objects are compiled in parallel and linked into
libfleet.so next to this file.
"""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_PKG = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_PKG, "csrc")
_OBJ = os.path.join(_PKG, "_build")
LIB_PATH = os.path.join(_PKG, "libfleet.so")
N_VARIANTS = 7
_DEPS = [os.path.join(_CSRC, n) for n in ("fleet.hip", "graph.cpp", "kernel_variant.hip", "kernels.hip.inc",
                                          "aux_kernels.hip.inc", "graph.hpp")] + \
        [os.path.join(_PKG, "..", "include", "fleet.h")]

_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
          # packed-FP32 instructions are not to be generated on the test machines
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wno-unused-value"]


def compile_jobs(extra=()) -> list:
    """(object path, hipcc command) of every translation unit."""
    jobs = [(os.path.join(_OBJ, "fleet.o"), ["hipcc", *_FLAGS, *extra, "-c", os.path.join(_CSRC, "fleet.hip")]),
            (os.path.join(_OBJ, "graph.o"), ["hipcc", *_FLAGS, *extra, "-x", "hip", "-c", os.path.join(_CSRC, "graph.cpp")])]
    for v in range(N_VARIANTS):
        jobs.append((os.path.join(_OBJ, f"variant{v}.o"),
                     ["hipcc", *_FLAGS, *extra, f"-DFLEET_VARIANT={v}", "-c", os.path.join(_CSRC, "kernel_variant.hip")]))
    return [(o, cmd + ["-o", o]) for o, cmd in jobs]


def build(force: bool = True, verbose: bool = False, jobs: int = 8, extra=()) -> str:
    """Compile libfleet.so in-tree.  With force=False an up-to-date library is kept."""
    if not force and os.path.exists(LIB_PATH) and \
            all(os.path.getmtime(LIB_PATH) >= os.path.getmtime(d) for d in _DEPS):
        return LIB_PATH
    os.makedirs(_OBJ, exist_ok=True)
    todo = compile_jobs(extra)

    def run(job):
        return subprocess.run(job[1], capture_output=True, text=True)

    with ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
        results = list(pool.map(run, todo))
    for (obj, cmd), res in zip(todo, results):
        if res.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + res.stdout + res.stderr)
        if verbose:
            print(res.stderr)
    link = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + [o for o, _ in todo]
    res = subprocess.run(link, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stdout + res.stderr)
    return LIB_PATH
