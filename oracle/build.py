"""Compile the CPU oracle (plain C, gcc) into oracle/libbs_oracle.so.

TEST INFRASTRUCTURE: the oracle checks the HIP path and is never part of it.
"""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "bs_oracle.c")
LIB = os.path.join(HERE, "libbs_oracle.so")

# -ffp-contract=off: the only fused multiply-add is the explicit fmaf() of the
# BatchNorm definition; no other a*b+c may be contracted behind our back.
CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
          "-fno-fast-math", "-fvisibility=hidden", "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.run(["gcc", *CFLAGS, SRC, "-o", tmp, "-lm"], check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build())
