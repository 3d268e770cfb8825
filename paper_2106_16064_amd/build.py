"""Builds ``libdgsp.so`` (HIP, gfx950) in place next to this file.

Run as ``python -m paper_2106_16064_amd.build``.  hipcc cross-compiles without
a GPU, so this works on any machine with ROCm installed.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from pathlib import Path

HERE = Path(__file__).resolve().parent
CSRC = HERE / "csrc"
LIB = HERE / "libdgsp.so"
SOURCES = [CSRC / "dgsp.hip"]
HEADERS = [CSRC / "dgsp_device.hpp", CSRC / "dgsp_kernels.hpp", HERE.parent / "include" / "dgsp.h"]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-munsafe-fp-atomics",                                      # native global_atomic_add_f32
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # no packed-fp32 instruction forms
    "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; libdgsp cannot be built")
    return exe


def build(verbose: bool = True, extra_flags=()) -> Path:
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-o", str(LIB), *map(str, SOURCES)]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the packed-fp32 feature and says so; that is expected
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return LIB


EXAMPLE_SRC = HERE.parent / "tests" / "c_abi_example.c"
EXAMPLE = HERE.parent / "tests" / "c_abi_example"


def build_c_example(verbose: bool = True) -> Path:
    """A plain-C caller of the library (gcc, no C++; a test program that lives under tests/): exercises the
    C-ABI from outside Python."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c11", "-O2", "-D__HIP_PLATFORM_AMD__", f"-I{rocm}/include", "-o", str(EXAMPLE), str(EXAMPLE_SRC),
           f"-L{HERE}", "-ldgsp", f"-L{rocm}/lib", "-lamdhip64", "-Wl,-rpath,$ORIGIN/../paper_2106_16064_amd", f"-Wl,-rpath,{rocm}/lib", "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"gcc failed on the C example:\n{res.stderr}")
    return EXAMPLE


def is_stale() -> bool:
    if not LIB.exists():
        return True
    t = LIB.stat().st_mtime
    return any(f.stat().st_mtime > t for f in SOURCES + HEADERS)


if __name__ == "__main__":
    build()
    build_c_example()
