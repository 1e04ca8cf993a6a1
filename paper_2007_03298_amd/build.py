"""Builds libdssync.so (HIP, gfx950 only) next to this file.

Run as ``python -m paper_2007_03298_amd.build``; the repository's build entry
point calls :func:`build_library`.  The shared object is kept in-tree so that
it travels with the sources to the GPU machine.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdssync.so")
SOURCES = ["partition.cpp", "pattern.cpp", "device_info.hip", "group_sync.hip", "consensus.hip"]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def compile_shared(sources, out: str, verbose: bool = False, extra_flags=()) -> str:
    """hipcc, gfx950 only, one shared object from the given sources."""
    cmd = [hipcc(), "-x", "hip", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Wall", "-Wno-unused-command-line-argument",
           # packed fp32 instructions are kept out of the generated code on purpose
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    cmd += list(extra_flags)
    cmd += list(sources)
    cmd += ["-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return out


def build_library(verbose: bool = False, extra_flags=(), out: str = LIB) -> str:
    return compile_shared([os.path.join(CSRC, s) for s in SOURCES], out, verbose, extra_flags)


if __name__ == "__main__":
    print(build_library(verbose=True))
