"""Compiles the HIP sources of this package for gfx950 into libcondensa.so (in-tree)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "api.hip")
LIB = os.path.join(HERE, "libcondensa.so")

FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                                   # one rounding per operation, as specified
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = list(FLAGS)
    if os.environ.get("CONDENSA_PLAIN_STREAM_STORES") == "1":
        # the compiler's own non-temporal stores instead of the buffer stores with system-scope bits: a build to
        # cross-check a parity failure against (csrc/common.h)
        flags.append("-DCONDENSA_PLAIN_STREAM_STORES")
    if os.environ.get("CONDENSA_INTEGER_F16") == "1":
        # binary16 rounding and widening in integer arithmetic throughout, instead of the conversion instructions
        flags.append("-DCONDENSA_INTEGER_F16")
    cmd = [hipcc] + flags + ["-o", LIB, SRC]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "packed-fp32-ops"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if verbose and err.strip():
        print(err)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
