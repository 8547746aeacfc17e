"""Compile the HIP sources of the library for gfx950 into libnsa_sel.so next to this file."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = ["api.hip", "index.hip", "fwd.hip", "bwd.hip", "select.hip", "qouter.hip", "profile.hip"]
LIB = os.path.join(HERE, "libnsa_sel.so")
# -packed-fp32-ops: keep the compiler from forming packed fp32 instructions
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wall"]


# The same sources with cycle stamps in the pipelined 128-key backward kernel (see pipe_timing.py): a measuring build,
# loaded by that module only.
LIB_TIMING = os.path.join(HERE, "libnsa_sel_timing.so")


def build(verbose: bool = False, timing: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = LIB_TIMING if timing else LIB
    cmd = [hipcc, *FLAGS, *(["-DNSA_PIPE_TIMING"] if timing else []), "-o", out,
           *[os.path.join(HERE, "csrc", s) for s in SOURCES]]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed")
    return out


if __name__ == "__main__":
    print(build(verbose=True))
    print(build(verbose=True, timing=True))
