"""Builds ``libdlion.so`` (the HIP kernels and their C ABI) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdlion.so")
SOURCES = [os.path.join(CSRC, "dlion.hip")]
HEADERS = [os.path.join(CSRC, "dlion_kernels.hpp"),
           os.path.join(os.path.dirname(HERE), "include", "dlion.h")]

# -ffp-contract=off: no multiply-add is ever fused (every fp32 operation rounds on its own).
# packed-fp32 ops are switched off for the whole library.
HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-ffp-contract=off", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    built = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > built for p in SOURCES + HEADERS)


def build(force: bool = False, verbose: bool = False) -> str:
    """Compile the library if it is missing, older than its sources, or ``force`` is set."""
    if force or is_stale():
        hipcc = os.environ.get("HIPCC", "hipcc")
        tmp = LIB + f".tmp{os.getpid()}"
        cmd = [hipcc, *HIPCC_FLAGS, "-o", tmp, *SOURCES]
        if verbose:
            print(" ".join(cmd), flush=True)
        proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if proc.returncode != 0:
            sys.stderr.write(proc.stdout)
            raise RuntimeError("hipcc failed building libdlion.so")
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
