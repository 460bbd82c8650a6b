"""Builds the HIP library (libnuts_hip.so) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libnuts_hip.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                      # a*b+c stays two roundings unless fma() is written out
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith(".hip")]


def headers():
    inc = os.path.join(os.path.dirname(HERE), "include")
    return [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith(".h")] + \
           [os.path.join(inc, f) for f in sorted(os.listdir(inc))]


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(p) > t for p in sources() + headers())


UBENCH_SRC = os.path.join(CSRC, "ubench", "issue_ubench.hip")
UBENCH_LIB = os.path.join(HERE, "libnuts_ubench.so")


def build(force: bool = True, verbose: bool = False) -> str:
    """The sampler library, and the instruction-issue microbenchmark as a library of its own."""
    if not force and not is_stale() and os.path.exists(UBENCH_LIB) and \
            os.path.getmtime(UBENCH_LIB) >= os.path.getmtime(UBENCH_SRC):
        return LIB_PATH
    for cmd in ([HIPCC] + FLAGS + sources() + ["-o", LIB_PATH], [HIPCC] + FLAGS + [UBENCH_SRC, "-o", UBENCH_LIB]):
        if verbose:
            print(" ".join(cmd), file=sys.stderr)
        subprocess.run(cmd, check=True)
    return LIB_PATH


if __name__ == "__main__":
    print(build(force=True, verbose=True))
