"""Build the HIP library (libpf_chain.so) in-tree for gfx950.

Every translation unit is compiled by hipcc with --offload-arch=gfx950 (cross-compiles without a GPU) and
with packed-fp32 instruction selection switched off; the objects are linked into
paper_2307_04995_amd/lib/libpf_chain.so, which is what the Python binding loads.

`python -m paper_2307_04995_amd.build --sanitize` builds a second library, lib/libpf_chain_san.so, whose HOST code
(description checking, lowering, recomposition, planning, merge plans, the C ABI) is instrumented with
AddressSanitizer and UndefinedBehaviorSanitizer (device code is left alone: GPU sanitizers are not available), builds
the C oracle the same way, and runs the CPU test suite (`pytest -m "not gpu"`) against the two.  CPU only.
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


# ---- host sanitizers -----------------------------------------------------------------------------------------------
HOST_SOURCES = ["pf_host.cpp", "pf_check.cpp", "pf_recompose.cpp", "pf_lower.cpp", "pf_plan.cpp", "pf_partition.cpp", "pf_jit.cpp",
                "pf_run_static.cpp"]
SAN_LIB = os.path.join(LIBDIR, "libpf_chain_san.so")
# each -fsanitize= directly behind -Xarch_host: the host pass only
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
             "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def _clang() -> str:
    return os.path.join(os.path.dirname(os.path.realpath(_hipcc())), "..", "llvm", "bin", "clang") \
        if os.path.exists(os.path.join(os.path.dirname(os.path.realpath(_hipcc())), "..", "llvm", "bin", "clang")) else "/opt/rocm/llvm/bin/clang"


def asan_runtime() -> str:
    out = subprocess.run([_clang(), "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True, check=True)
    return out.stdout.strip()


def build_sanitized(verbose: bool = False) -> tuple:
    """The library with instrumented host code, and the oracle built the same way.  Returns their paths."""
    if not is_built():
        build(force=True, verbose=verbose)   # the device objects are shared with the ordinary build
    hipcc = _hipcc()
    san_dir = os.path.join(OBJDIR, "san")
    os.makedirs(san_dir, exist_ok=True)

    def compile_host(src: str) -> str:
        obj = os.path.join(san_dir, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc] + [f for f in FLAGS if f != "-O3"] + ["-O1"] + SAN_FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            sys.stderr.write(res.stdout + res.stderr)
            raise RuntimeError(f"hipcc failed on {src}")
        return obj

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        host_objs = list(pool.map(compile_host, HOST_SOURCES))
    dev_objs = [os.path.join(OBJDIR, os.path.splitext(s)[0] + ".o") for s in SOURCES if s not in HOST_SOURCES]
    missing = [o for o in dev_objs if not os.path.exists(o)]
    if missing:
        build(force=True, verbose=verbose)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined", "-shared-libsan",
           "-Wl,--version-script=" + os.path.join(CSRC, "pf_chain.map"), "-o", SAN_LIB] + host_objs + dev_objs + ["-lhiprtc", "-ldl"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("link of the sanitized library failed")
    root = os.path.dirname(HERE)
    oracle_san = os.path.join(root, "oracle", "libpf_oracle_san.so")
    cmd = [_clang(), "-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined",
           "-shared-libsan", "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-o", oracle_san, os.path.join(root, "oracle", "pf_oracle.c"), "-lm"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("build of the sanitized oracle failed")
    return SAN_LIB, oracle_san


def run_sanitized_tests(extra_args=()) -> int:
    """pytest -m "not gpu" against the instrumented library and oracle.  The interpreter is not instrumented, so the
    sanitizer run time is preloaded (in front of whatever is preloaded already)."""
    lib, oracle_lib = build_sanitized()
    env = dict(os.environ)
    pre = [asan_runtime()] + [p for p in env.get("LD_PRELOAD", "").split(":") if p]
    env["LD_PRELOAD"] = ":".join(pre)
    # (reports go to files: a report ends the process, and with it whatever pytest had captured)
    import glob
    import tempfile
    log_dir = tempfile.mkdtemp(prefix="pf_san_")
    env["ASAN_OPTIONS"] = f"detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:halt_on_error=1:log_path={log_dir}/asan"
    env["UBSAN_OPTIONS"] = f"print_stacktrace=1:halt_on_error=1:log_path={log_dir}/ubsan"
    env["PF_CHAIN_LIB"] = lib
    env["PF_ORACLE_LIB"] = oracle_lib
    root = os.path.dirname(HERE)
    cmd = [sys.executable, "-m", "pytest", os.path.join(root, "tests"), "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + list(extra_args)
    rc = subprocess.run(cmd, env=env, cwd=root).returncode
    for path in sorted(glob.glob(os.path.join(log_dir, "*"))):
        with open(path) as fh:
            sys.stderr.write(f"---- {os.path.basename(path)}\n" + fh.read()[:20000])
        rc = rc or 1
    return rc


if __name__ == "__main__":
    if "--sanitize" in sys.argv[1:]:
        sys.exit(run_sanitized_tests([a for a in sys.argv[1:] if a != "--sanitize"]))
    print(build(force=True, verbose=True))
