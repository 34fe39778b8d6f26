"""Build libbrainslug_hip.so (hipcc, gfx950) in-tree, next to this file."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libbrainslug_hip.so")
SOURCES = ["bs_stack.cpp", "bs_plan.cpp", "bs_run.cpp", "bs_kernels.hip", "bs_lds.hip", "bs_rows.hip", "bs_rows2.hip"]

# -ffp-contract=off: the only fused multiply-add is the explicit one of BatchNorm.
# packed-fp32 instructions are disabled for the device code.
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-ffp-contract=off",
         "-fno-fast-math", "-fvisibility=hidden", "-Wall", "-Wextra", "-Wno-unused-parameter",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # the by-value kernel argument blocks are read in place (kernarg segment) only if the
         # optimizer may look through all their uses; the default cap is too low for the LDS kernel
         "-mllvm", "-instcombine-max-copied-from-constant-users=100000",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def up_to_date() -> bool:
    if not os.path.exists(LIB):
        return False
    t = os.path.getmtime(LIB)
    deps = sources() + [os.path.join(CSRC, "bs_internal.h"), os.path.join(CSRC, "bs_device.h"), os.path.join(ROOT, "include", "brainslug.h")]
    return all(os.path.getmtime(d) <= t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and up_to_date():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in FLAGS if f != "-shared"]

    def compile_one(src):
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        cmd = [hipcc, *compile_flags, "-x", "hip", "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True)
        return obj

    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, sources()))
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fvisibility=hidden", *objs, "-o", tmp],
                   check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
