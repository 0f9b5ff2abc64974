"""Build step: compile the HIP sources into ``libgemm_epilogue.so`` (the operator) and
``libge_probes.so`` (the measurement probes) for gfx950.

``python -m paper_2604_01489_amd.build`` or ``build_library()``.  hipcc cross
compiles without a GPU.  The library is kept in-tree, next to this file.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgemm_epilogue.so")
PROBES_LIB = os.path.join(HERE, "libge_probes.so")
# the longest compiles first (the pool takes the sources in this order)
LIB_SOURCES = ["conv_halo_14_11.hip", "conv_halo_12_12.hip", "conv_api.hip", "gemm_fused_t256.hip", "gemm_fused_t256_edge.hip", "gemm_fused_t128.hip", "gemm_fused_t128_edge.hip",
               "gemm_fused_w4_e0.hip", "gemm_fused_w4_e1.hip", "gemm_fused_w4_e2.hip", "gemm_epilogue_api.hip",
               "gemm_fused_api.hip", "gemm_symm_api.hip", "gemm_diag.hip", "gemm_rowsum.hip"]
PROBE_SOURCES = ["ge_probes.hip"]
SOURCES = LIB_SOURCES + PROBE_SOURCES
# packed fp32 instructions are kept off: some of their forms have misbehaved on this hardware
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _includes(path, seen):
    """Files a source pulls in through #include "..." (transitively)."""
    import re
    if path in seen or not os.path.exists(path):
        return seen
    seen.add(path)
    for inc in re.findall(r'^\s*#include\s+"([^"]+)"', open(path).read(), flags=re.M):
        _includes(os.path.normpath(os.path.join(os.path.dirname(path), inc)), seen)
    return seen


def build_library(verbose: bool = False, extra_flags=(), incremental: bool = False) -> str:
    """Compile every source to an object (in parallel: the kernel templates dominate the build
    time), then link the two libraries.  ``incremental`` keeps the objects that are newer than
    the source and every header it includes (for work on one file; the default compiles all)."""
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in FLAGS if f != "-shared"]

    def compile_one(src):
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        if incremental and not extra_flags and os.path.exists(obj):
            deps = _includes(os.path.join(CSRC, src), set())
            if all(os.path.getmtime(d) <= os.path.getmtime(obj) for d in deps):
                return obj
        cmd = ["hipcc", *compile_flags, *extra_flags, "-c", "-o", obj, os.path.join(CSRC, src)]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            sys.stderr.write(res.stdout + res.stderr)
            raise RuntimeError(f"hipcc failed on {src}")
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    n = len(LIB_SOURCES)
    for out, group in ((LIB, objs[:n]), (PROBES_LIB, objs[n:])):
        cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *group]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            sys.stderr.write(res.stdout + res.stderr)
            raise RuntimeError("link failed")
    return LIB


def library_is_current() -> bool:
    if not os.path.exists(LIB) or not os.path.exists(PROBES_LIB):
        return False
    t = min(os.path.getmtime(LIB), os.path.getmtime(PROBES_LIB))
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    inc = os.path.join(os.path.dirname(HERE), "include")
    deps += [os.path.join(inc, f) for f in os.listdir(inc)]
    return all(os.path.getmtime(d) <= t for d in deps)


if __name__ == "__main__":
    print(build_library(verbose=True, incremental="--incremental" in sys.argv[1:]))
