"""Builds libsketch_linear.so (HIP, gfx950 only) in-tree with hipcc.

Every source file is one translation unit; they are compiled side by side
into `_build/` at the repository root and linked into the shared library.
"""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(ROOT, "_build")
LIB = os.path.join(HERE, "libsketch_linear.so")
# the same library with range asserts in its kernels (-DSKL_DEBUG_BOUNDS): violations are counted, not trapped
DEBUG_LIB = os.path.join(HERE, "libsketch_linear_debug.so")
# compiled once
COMMON_SOURCES = ["skl_host.cpp", "skl_file.cpp", "skl_dispatch.cpp", "skl_lowbit.hip", "skl_build.hip", "skl_microbench.hip"]
# compiled once per query mode (-DSKL_QM=0 / 1): their kernels and launchers live in a namespace per mode
MODE_SOURCES = ["skl_prefill.hip", "skl_decode.hip", "skl_prefill_staged.hip", "skl_reconstruct.hip", "skl_tile.hip",
                "skl_naive.hip"]
SOURCES = COMMON_SOURCES + MODE_SOURCES


def lib_path() -> str:
    """The built library; SKETCH_LINEAR_LIB names another build to load instead (the host-only sanitizer
    build of the test suite)."""
    return os.environ.get("SKETCH_LINEAR_LIB") or LIB


def _flags():
    return ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-x", "hip",
            # packed-fp32 VALU forms are kept out of the generated code
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wno-unused-command-line-argument", "-Wno-ignored-attributes", "-Wno-inline-asm",
            "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (res.stdout + res.stderr).splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def _stale(src: str, obj: str) -> bool:
    if not os.path.exists(obj):
        return True
    deps = [src] + [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    deps += [os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include"))]
    return any(os.path.getmtime(d) > os.path.getmtime(obj) for d in deps)


def build_library(verbose: bool = False, jobs: int | None = None, incremental: bool = False, debug_bounds: bool = False) -> str:
    """Compile every source for gfx950 and link the shared library.  With
    `incremental`, objects newer than their source and every header are kept.
    `debug_bounds` builds the variant whose kernels carry range asserts."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    obj_dir = os.path.join(OBJ_DIR, "debug") if debug_bounds else OBJ_DIR
    os.makedirs(obj_dir, exist_ok=True)
    jobs = jobs or max(1, min(os.cpu_count() or 1, 8))
    extra = ["-DSKL_DEBUG_BOUNDS"] if debug_bounds else []
    units = [(s, extra, os.path.splitext(s)[0] + ".o") for s in COMMON_SOURCES]
    # the long compilations first, so that the pool ends evenly
    units = [(s, extra + [f"-DSKL_QM={m}"], f"{os.path.splitext(s)[0]}_qm{m}.o") for s in MODE_SOURCES for m in (0, 1)] + units
    objs = [os.path.join(obj_dir, o) for _, _, o in units]
    cmds = [[hipcc] + _flags() + defs + ["-c", os.path.join(CSRC, s), "-o", o] for (s, defs, _), o in zip(units, objs)
            if not incremental or _stale(os.path.join(CSRC, s), o)]
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        list(pool.map(lambda c: _run(c, verbose), cmds))
    lib = DEBUG_LIB if debug_bounds else LIB
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fvisibility=hidden"] + objs + ["-o", lib], verbose)
    return lib


if __name__ == "__main__":
    import sys
    print(build_library(verbose=True, incremental="--incremental" in sys.argv, debug_bounds="--debug-bounds" in sys.argv))
