"""Builds libtuna.so (the HIP kernels + the C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import hashlib
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtuna.so")
SOURCES = [os.path.join(CSRC, "tuna_api.hip")]
HEADERS = [os.path.join(CSRC, "tuna_kernels.h"), os.path.join(CSRC, "tuna_plan.h"),
           os.path.join(os.path.dirname(HERE), "include", "tuna.h")]


def source_hash() -> str:
    """Hash of every source and header the library is built from; compiled into the library
    (tuna_build_id) so that a loaded library can be told from one built from other sources."""
    h = hashlib.sha256()
    for f in SOURCES + HEADERS:
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def hipcc_command(out: str) -> list:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    return [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
            "-DTUNA_BUILD_ID=\"%s\"" % source_hash(),
            # packed-FP32 instructions are not wanted in any code object of this library
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wall", "-Wno-unused-function", "-Wno-unused-command-line-argument",
            "-o", out] + SOURCES


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compile the library (always when force=True; else only when sources are newer)."""
    if not force and not is_stale():
        return LIB
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = hipcc_command(tmp)
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise RuntimeError("hipcc failed:\n" + proc.stdout)
    if verbose and proc.stdout.strip():
        print(proc.stdout, file=sys.stderr)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
