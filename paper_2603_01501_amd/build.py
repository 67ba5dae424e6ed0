"""Builds libgac.so (HIP kernels + C ABI) for gfx950, in-tree, with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
LIB_PATH = os.path.join(_PKG, "libgac.so")
SOURCES = [os.path.join(_PKG, "csrc", "gac_kernels.hip"), os.path.join(_PKG, "csrc", "gac_api.cpp")]
HEADERS = [os.path.join(_PKG, "csrc", "gac_internal.h"), os.path.join(_ROOT, "include", "gac.h")]

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 instructions are kept off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(_ROOT, "include"), "-I", os.path.join(_PKG, "csrc"),
]


def source_hash() -> str:
    """SHA-256 over the bytes of every source and header the library is built from.  The build
    compiles it into the library (gac_source_hash()), and the binding refuses a library whose
    hash is not that of the sources next to it: a stale binary is an error, never a silent
    stand-in."""
    import hashlib
    h = hashlib.sha256()
    for f in SOURCES + HEADERS:
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ['-DGAC_SOURCE_HASH="%s"' % source_hash()] + SOURCES + ["-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("hipcc failed building libgac.so")
    if verbose and (r.stdout or r.stderr):
        print(r.stdout + r.stderr)
    return LIB_PATH


def kernel_code_sha256() -> str:
    """SHA-256 of the kernel source with // comments and blank lines removed: changes when the
    code of a kernel changes, not when a comment does.  The counter summaries under profiles/
    record it, and the benchmark reports their traffic figure only while it still matches."""
    import hashlib
    import re
    lines = []
    with open(SOURCES[0]) as f:
        for line in f:
            line = re.sub(r"//.*$", "", line).rstrip()
            if line.strip():
                lines.append(line)
    return hashlib.sha256("\n".join(lines).encode()).hexdigest()


C_CHECK_SRC = os.path.join(_ROOT, "tests", "c_abi_check.cpp")
C_CHECK_BIN = os.path.join(_ROOT, "tests", "c_abi_check.bin")


def build_c_abi_check(verbose: bool = False) -> str:
    """A plain C++ program that calls libgac.so without Python or PyTorch (used by a GPU test)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O2", "-std=c++17", "-Wall", "-Wno-unused-command-line-argument",
           "-I", os.path.join(_ROOT, "include"), C_CHECK_SRC, "-o", C_CHECK_BIN,
           "-L", _PKG, "-l:libgac.so", "-Wl,-rpath," + _PKG, "-Wl,-rpath,$ORIGIN/../paper_2603_01501_amd"]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("hipcc failed building tests/c_abi_check.bin")
    return C_CHECK_BIN


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_c_abi_check(verbose=True))
