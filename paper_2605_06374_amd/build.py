"""Compile csrc/varlen_attn.hip (with the .hpp files it includes) for gfx950 into libvarlen_attn.so,
csrc/varlen_attn_bench.hip (measurement probes) into libvarlen_attn_bench.so, and the host-only
csrc/mb_time.cpp, csrc/pipeline_dag.cpp, csrc/tp_select.cpp, csrc/migration_step.cpp and
csrc/migration_plan.cpp into
shared libraries of the same names, next to this file."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "varlen_attn.hip")
LIB = os.path.join(HERE, "libvarlen_attn.so")
# measurement probes for bench.py only (matrix-pipe and LDS rates); not part of the library's ABI
BENCH_SRC = os.path.join(HERE, "csrc", "varlen_attn_bench.hip")
BENCH_LIB = os.path.join(HERE, "libvarlen_attn_bench.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-I" + os.path.join(ROOT, "include"),
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # uniform-address LDS atomics from a few lanes: the optimizer's lane-by-lane reduction
    # loop costs far more than the atomic it saves
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
    # the hand-placed instruction order of the inner loops is kept after register allocation
    "-mllvm", "-enable-post-misched=0",
    "-Wno-unused-command-line-argument",
]


# host-only libraries: the Detector's predictors of Section 5.2, the Scheduler's TP subgroup
# selection of Section 6.1 and migration decision of Section 6.3
HOST_LIBS = {"libmb_time.so": "mb_time.cpp", "libpipeline_dag.so": "pipeline_dag.cpp",
             "libtp_select.so": "tp_select.cpp", "libmigration_step.so": "migration_step.cpp",
             "libmigration_plan.so": "migration_plan.cpp migration_step.cpp"}


def build_host(verbose: bool = False) -> list:
    out = []
    for lib, src in HOST_LIBS.items():
        cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-I" + os.path.join(ROOT, "include"), "-o", os.path.join(HERE, lib)] + \
              [os.path.join(HERE, "csrc", f) for f in src.split()]
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True)
        out.append(os.path.join(HERE, lib))
    return out


def build(verbose: bool = False) -> str:
    build_host(verbose)
    for lib, src in ((BENCH_LIB, BENCH_SRC), (LIB, SRC)):
        cmd = [HIPCC] + FLAGS + ["-o", lib, src]
        if verbose:
            print(" ".join(cmd))
        res = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + err)
        if verbose and err.strip():
            print(err)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
