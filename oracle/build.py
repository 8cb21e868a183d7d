"""Compile the CPU oracle (plain C, gcc) into oracle/liborc.so.  Test infrastructure only."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "actorq_oracle.c")
LIB = os.path.join(HERE, "liborc.so")


def build(force: bool = True, src: str = SRC, lib: str = LIB) -> str:
    """Compiles `src` into `lib` (defaults: the oracle itself; the mutation test passes altered copies)."""
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(src):
        return lib
    # -ffp-contract=off: no fused multiply-add may replace the written fp32/fp64 operations
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wextra", "-o", lib, src, "-lm"]
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build())
