"""Build step of the HIP library: one hipcc invocation, gfx950 only.

    python -m paper_1901_01544_amd.build

The shared object is written next to this file (``libiwp.so``), in-tree, so it
travels with the source tree to wherever the GPU is.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "iwp_api.hip")
LIB = os.path.join(HERE, "libiwp.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-shared",
    # IEEE binary32 as the method is defined: no contraction, no fast-math,
    # denormals kept, correctly rounded divide.
    "-ffp-contract=off",
    "-fno-fast-math",
    "-fno-gpu-flush-denormals-to-zero",
    "-fhip-fp32-correctly-rounded-divide-sqrt",
    # packed fp32 instructions stay off on these machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def build(verbose: bool = False, extra_flags=(), out: str = LIB) -> str:
    """Compile csrc/ into libiwp.so (always recompiles); returns the path.
    extra_flags / out: build a tuning variant (e.g. -DIWP_LGROUP=4) somewhere else."""
    tmp = out + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-o", tmp, SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
