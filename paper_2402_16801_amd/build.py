"""Compiles the HIP library in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
SRCS = [os.path.join(_PKG, "csrc", f) for f in ("craftax.hip", "full.hip")]
OUT = os.path.join(_PKG, "libcraftax_hip.so")

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                                         # floats are single IEEE ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # no packed-fp32 instructions
]


DEBUG_OUT = os.path.join(_PKG, "libcraftax_hip_debug.so")


def build_library(verbose: bool = False, only_changed: bool = False, debug_bounds: bool = False) -> str:
    """Compiles every translation unit (in parallel) and links the library.  only_changed skips a
    unit whose object is newer than every source and header (for quick iteration; the build check
    always compiles everything)."""
    from concurrent.futures import ThreadPoolExecutor

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(_PKG, "_build_debug" if debug_bounds else "_build")
    os.makedirs(objdir, exist_ok=True)
    csrc = os.path.join(_PKG, "csrc")
    deps = [os.path.join(csrc, f) for f in os.listdir(csrc)] + [os.path.join(os.path.dirname(_PKG), "include", "craftax.h")]
    newest = max(os.path.getmtime(d) for d in deps)
    flags = [f for f in HIPCC_FLAGS if f != "-shared"] + (["-DCRAFTAX_DEBUG_BOUNDS"] if debug_bounds else [])
    out = DEBUG_OUT if debug_bounds else OUT

    def compile_one(src):
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        if only_changed and os.path.exists(obj) and os.path.getmtime(obj) >= newest:
            return obj
        cmd = [hipcc] + flags + ["-c", "-o", obj, src]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + res.stderr)
        if verbose:
            print(" ".join(cmd))
        return obj

    with ThreadPoolExecutor(max_workers=len(SRCS)) as ex:
        objs = list(ex.map(compile_one, SRCS))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out] + objs
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc link failed:\n" + res.stderr)
    if verbose:
        print(" ".join(cmd))
    return out


def build_all(only_changed: bool = False):
    """The release library and the bounds-checking debug library, side by side."""
    from concurrent.futures import ThreadPoolExecutor

    with ThreadPoolExecutor(max_workers=2) as ex:
        a = ex.submit(build_library, False, only_changed, False)
        b = ex.submit(build_library, False, only_changed, True)
        return a.result(), b.result()


EXAMPLE_SRC = os.path.join(os.path.dirname(_PKG), "examples", "step_from_c.c")
EXAMPLE_OUT = os.path.join(os.path.dirname(_PKG), "examples", "step_from_c")


def build_example() -> str:
    """The plain-C consumer of the ABI: gcc, the HIP runtime and the library, nothing else."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-O2", "-std=c11", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"), "-o", EXAMPLE_OUT, EXAMPLE_SRC,
           "-L", _PKG, "-l:libcraftax_hip.so", "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../paper_2402_16801_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("gcc failed:\n" + res.stderr)
    return EXAMPLE_OUT


if __name__ == "__main__":
    print(build_all())
    print(build_example())
