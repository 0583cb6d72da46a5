"""Build the HIP library (libkdn.so) for gfx950, in tree, with hipcc."""
from __future__ import annotations

import hashlib
import os
import re
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
SOURCES = [os.path.join(_PKG, "csrc", "kdn.hip"), os.path.join(_PKG, "csrc", "kdn_arena.hip"),
           os.path.join(_PKG, "csrc", "kdn_pool.cpp")]
HEADERS = [os.path.join(_ROOT, "include", "kdn.h"), os.path.join(_ROOT, "include", "kdn_pool.h"),
           os.path.join(_ROOT, "include", "kdn_arena.h"),
           os.path.join(_PKG, "csrc", "kdn_kernels.h"), os.path.join(_PKG, "csrc", "kdn_planner.h"),
           os.path.join(_PKG, "csrc", "kdn_blocklist.h")]
LIB_PATH = os.path.join(_PKG, "libkdn.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                 # products and fused multiply-adds exactly as written
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
]


def source_fingerprint(files=None) -> str:
    """sha256 (first 16 hex digits) over the library's sources, headers and compiler flags.
    It is compiled into the library (kdn_version() ends with it), so that a binary can be
    matched against the sources beside it."""
    h = hashlib.sha256()
    for f in (SOURCES + HEADERS) if files is None else files:
        h.update(os.path.basename(f).encode() + b"\0")
        with open(f, "rb") as fh:
            h.update(fh.read())
        h.update(b"\0")
    h.update(" ".join(HIPCC_FLAGS).encode())
    return h.hexdigest()[:16]


_MARK = re.compile(rb"kdn-gfx950 [0-9.]+ src:([0-9a-f]{16})")


def library_fingerprint(path=None):
    """The source fingerprint a built library carries (read from the file, nothing is
    loaded), or None if there is no library or it carries none."""
    path = LIB_PATH if path is None else path
    if not os.path.exists(path):
        return None
    with open(path, "rb") as fh:
        m = _MARK.search(fh.read())
    return m.group(1).decode() if m else None


def is_stale(path=None, files=None) -> bool:
    """True when there is no library or it was built from other sources or flags."""
    return library_fingerprint(path) != source_fingerprint(files)


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compile csrc/*.hip into libkdn.so.  hipcc cross-compiles; no GPU is needed."""
    if not force and not is_stale():
        return LIB_PATH
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB_PATH + ".%d.tmp" % os.getpid()
    cmd = ([hipcc] + HIPCC_FLAGS + ["-DKDN_SRC_HASH=\"%s\"" % source_fingerprint(),
                                    "-I", os.path.join(_ROOT, "include"), "-o", tmp] + SOURCES)
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
    """The library that matches the sources in the tree: built when there is none, built
    again when the one that is there carries another source fingerprint.  A failing
    compiler raises; a stale binary is never handed out."""
    if is_stale():
        build_library(force=True)
        if is_stale():
            raise RuntimeError("libkdn.so does not carry the fingerprint of the sources it was just built from")
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
