"""Build the HIP library (libpf_chain.so) in-tree for gfx950.

Every translation unit is compiled by hipcc with --offload-arch=gfx950 (cross-compiles without a GPU) and
with packed-fp32 instruction selection switched off; the objects are linked into
paper_2307_04995_amd/lib/libpf_chain.so, which is what the Python binding loads.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIBDIR = os.path.join(HERE, "lib")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(LIBDIR, "libpf_chain.so")

SOURCES = ["pf_host.cpp", "pf_check.cpp", "pf_recompose.cpp", "pf_lower.cpp", "pf_plan.cpp", "pf_partition.cpp", "pf_jit.cpp", "pf_run_static.cpp", "pf_row_generic.hip", "pf_row_stream.hip", "pf_row_static.hip", "pf_row_static_f32.hip", "pf_row_static_f16.hip",
           "pf_row_static_bf16.hip", "pf_perm.hip", "pf_group.hip", "pf_attn.hip", "pf_gather.hip", "pf_stencil.hip", "pf_pool.hip", "pf_col.hip", "pf_cast.hip"]
HEADERS = ["pf_common.h", "pf_host_internal.h", "pf_chain.map", "pf_device.hpp", "pf_jit.h", "pf_launch.h", "pf_row_kernels.hpp", "pf_row_stream.hpp", "pf_perm_kernels.hpp", "pf_group_kernels.hpp", "pf_stencil_kernels.hpp", "pf_pool_kernels.hpp", "pf_col_kernels.hpp", "pf_specs.h", "pf_row_static.inc",
           os.path.join("..", "..", "include", "pf_chain.h")]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-pass-failed",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-x", "hip"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _newest_input() -> float:
    paths = [os.path.join(CSRC, s) for s in SOURCES] + [os.path.normpath(os.path.join(CSRC, h)) for h in HEADERS]
    return max(os.path.getmtime(p) for p in paths)


def is_built() -> bool:
    return os.path.exists(LIB)


def is_fresh() -> bool:
    return is_built() and os.path.getmtime(LIB) >= _newest_input()


def build(force: bool = True, verbose: bool = False, jobs: int | None = None) -> str:
    """Compile every source and link the shared library.  Returns its path."""
    if not force and is_fresh():
        return LIB
    os.makedirs(LIBDIR, exist_ok=True)
    os.makedirs(OBJDIR, exist_ok=True)
    hipcc = _hipcc()
    jobs = jobs or min(len(SOURCES), max(1, min(16, os.cpu_count() or 1)))

    def compile_one(src: str) -> str:
        obj = os.path.join(OBJDIR, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            sys.stderr.write(res.stdout + res.stderr)
            raise RuntimeError(f"hipcc failed on {src}")
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-Wl,--version-script=" + os.path.join(CSRC, "pf_chain.map"), "-o", LIB] + objs + ["-lhiprtc", "-ldl"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("link failed")
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
