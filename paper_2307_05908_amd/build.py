"""Build libppd.so for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libppd.so")
SOURCES = [os.path.join(HERE, "csrc", "ppd_engine.hip")]
DEPS = SOURCES + [os.path.join(HERE, "csrc", "ppd_kernels.h"),
                  os.path.join(os.path.dirname(HERE), "include", "ppd.h")]
# -ffp-contract=off: every fused multiply-add in the kernels is an explicit fmaf, so a row's arithmetic
# does not depend on which template instance it runs in.  Packed-fp32 code generation is switched off.
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-variable"]


def stale() -> bool:
    return (not os.path.exists(LIB_PATH)) or any(os.path.getmtime(LIB_PATH) < os.path.getmtime(s) for s in DEPS)


def build(force: bool = True, verbose: bool = False) -> str:
    if force or stale():
        cmd = ["hipcc"] + FLAGS + ["-o", LIB_PATH] + SOURCES
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
    return LIB_PATH


if __name__ == "__main__":
    print(build(True, True))
