"""Build the HIP library (libkdn.so) for gfx950, in tree, with hipcc."""
from __future__ import annotations

import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
SOURCES = [os.path.join(_PKG, "csrc", "kdn.hip"), os.path.join(_PKG, "csrc", "kdn_pool.cpp")]
HEADERS = [os.path.join(_ROOT, "include", "kdn.h"), os.path.join(_ROOT, "include", "kdn_pool.h"),
           os.path.join(_PKG, "csrc", "kdn_kernels.h"), os.path.join(_PKG, "csrc", "kdn_planner.h")]
LIB_PATH = os.path.join(_PKG, "libkdn.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                 # products and fused multiply-adds exactly as written
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
]


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS + [os.path.abspath(__file__)])


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compile csrc/*.hip into libkdn.so.  hipcc cross-compiles; no GPU is needed."""
    if not force and not is_stale():
        return LIB_PATH
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB_PATH + ".%d.tmp" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + ["-I", os.path.join(_ROOT, "include"), "-o", tmp] + SOURCES
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout + proc.stderr)
    # hipcc's host pass does not know the packed-fp32 target feature and says so; anything else is shown
    noise = ("packed-fp32-ops", "warning generated", "warnings generated")
    for line in (proc.stdout + proc.stderr).splitlines():
        if line.strip() and not any(n in line for n in noise):
            print(line, flush=True)
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


def ensure_built() -> str:
    """Build only when no library is there at all (a fresh checkout); one that is there is
    used as it is."""
    return LIB_PATH if os.path.exists(LIB_PATH) else build_library(force=True)


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
