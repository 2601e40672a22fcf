"""Builds libsvip.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = [os.path.join(HERE, "csrc", "svip_kernels.hip"), os.path.join(HERE, "csrc", "svip_loop.hip")]
HEADERS = sorted(os.path.join(HERE, "csrc", f) for f in os.listdir(os.path.join(HERE, "csrc")) if f.endswith(".h")) + \
    [os.path.join(ROOT, "include", "svip.h")]
LIB = os.path.join(HERE, "libsvip.so")
EXAMPLE_SRC = os.path.join(HERE, "examples", "round_from_file.cpp")
EXAMPLE_BIN = os.path.join(HERE, "examples", "round_from_file")

# packed-fp32 instructions are switched off for all device code of this library
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"),
]


def build(verbose: bool = False) -> str:
    """Compile every HIP source of the package; returns the library path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [hipcc, *HIPCC_FLAGS, *SOURCES, "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines()
                    if "is not a recognized feature for this target" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    os.replace(tmp, LIB)
    build_example(verbose)
    return LIB


def build_example(verbose: bool = False) -> str:
    """The C-ABI example program (plain HIP host code linked against libsvip.so, found at run time
    through an rpath relative to the executable)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = EXAMPLE_BIN + f".tmp{os.getpid()}"
    cmd = [hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-I" + os.path.join(ROOT, "include"), EXAMPLE_SRC,
           "-L" + HERE, "-lsvip", "-Wl,-rpath,$ORIGIN/..", "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed on the example:\n" + proc.stdout)
    os.replace(tmp, EXAMPLE_BIN)
    return EXAMPLE_BIN


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    if not os.path.exists(EXAMPLE_BIN):
        return True
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS + [EXAMPLE_SRC])


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
