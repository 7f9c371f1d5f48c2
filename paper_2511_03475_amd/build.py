"""Builds libcp_extend.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
SOURCES = [os.path.join(_PKG, "csrc", "cp_extend.hip"),
           os.path.join(_PKG, "csrc", "cp_context_distance.hip"),
           os.path.join(_PKG, "csrc", "cp_probe.hip"),
           os.path.join(_PKG, "csrc", "cp_context_index.cpp"),
           os.path.join(_PKG, "csrc", "cp_context_dedup.cpp")]
INCLUDE = os.path.join(_ROOT, "include")
LIB_PATH = os.path.join(_PKG, "libcp_extend.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = False) -> str:
    """Compile every HIP source of the library for gfx950; returns the path of the .so."""
    cmd = [hipcc_path(), *HIPCC_FLAGS, "-I", INCLUDE, *SOURCES, "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
