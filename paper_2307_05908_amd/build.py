"""Build libppd.so for gfx950 with hipcc (cross-compiles without a GPU).

The kernel template instances are spread over several translation units (csrc/ppd_inst.hip with
-DPPD_INST=n) that compile in parallel; objects go to a scratch directory outside the tree.
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libppd.so")
PROBE_PATH = os.path.join(HERE, "ppd_pmc_probe")
N_INST = 7
DEPS = [os.path.join(CSRC, f) for f in ("ppd_engine.hip", "ppd_ops.hip", "ppd_pmc_probe.cpp", "ppd_prefill.hip", "ppd_prefill.h", "ppd_inst.hip", "ppd_kernels.h", "ppd_launch.h")] + \
       [os.path.join(os.path.dirname(HERE), "include", f) for f in ("ppd.h", "ppd_measure.h")]
# -ffp-contract=off: every fused multiply-add in the kernels is an explicit fmaf, so a row's arithmetic
# does not depend on which template instance it runs in.  Packed-fp32 code generation is switched off.
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-variable", "-Wno-inline-asm"]


def stale() -> bool:
    return (not os.path.exists(LIB_PATH)) or any(os.path.getmtime(LIB_PATH) < os.path.getmtime(s) for s in DEPS)


def _compile(args):
    src, obj, extra, verbose = args
    cmd = ["hipcc"] + FLAGS + extra + ["-c", src, "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src} {extra}:\n{out}")
    return out


def build(force: bool = True, verbose: bool = False, jobs: int = 0) -> str:
    if not (force or stale()):
        return LIB_PATH
    jobs = jobs or min(8, os.cpu_count() or 4)
    with tempfile.TemporaryDirectory(prefix="ppd_build_") as tmp:
        units = [(os.path.join(CSRC, "ppd_engine.hip"), os.path.join(tmp, "engine.o"), [], verbose),
                 (os.path.join(CSRC, "ppd_ops.hip"), os.path.join(tmp, "ops.o"), [], verbose),
                 (os.path.join(CSRC, "ppd_prefill.hip"), os.path.join(tmp, "prefill.o"), [], verbose)]
        for i in range(N_INST):
            units.append((os.path.join(CSRC, "ppd_inst.hip"), os.path.join(tmp, f"inst{i}.o"), [f"-DPPD_INST={i}"], verbose))
        with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
            for out in ex.map(_compile, units):
                if out.strip() and verbose:
                    print(out)
        cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + [u[1] for u in units]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        # the counter probe: a small program on the C ABI (no Python), for rocprofv3 --pmc runs
        cmd = ["hipcc", "-O2", "-std=c++17", "--offload-arch=gfx950", "-o", PROBE_PATH, os.path.join(CSRC, "ppd_pmc_probe.cpp"),
               "-L" + HERE, "-lppd", "-Wl,-rpath,$ORIGIN"]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
    return LIB_PATH


if __name__ == "__main__":
    print(build(True, True))
