"""Builds libmlpo.so (the C-ABI library of HIP kernels) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmlpo.so")
SOURCES = ["adamw.hip", "gradnorm.hip", "accum.hip", "api.hip", "pipeline.hip", "filetier.hip", "tiers.hip", "repack.hip"]

# -ffp-contract=off: every fp32 operation of the update rounds on its own (no fused multiply-add), which is what makes
# bit-level comparison with a plain CPU evaluation possible.  Division and square root stay IEEE-correct (hipcc's
# default) and denormals are kept.
HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-ffp-contract=off", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def hipcc() -> str:
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cand = os.path.join(rocm, "bin", "hipcc")
    return cand if os.path.exists(cand) else "hipcc"


def build_lib(verbose: bool = False, extra_flags=()) -> str:
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", LIB, *srcs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


YARDSTICK_SRC = os.path.join(ROOT, "bench_yardsticks.hip")
YARDSTICK_LIB = os.path.join(ROOT, "libbench_yardsticks.so")
YARDSTICK_EXE = os.path.join(ROOT, "bench_link_yardstick")


def build_yardsticks(verbose: bool = False) -> str:
    """The benchmark's measuring aid (bare memory sweeps, link copies): a shared object of its own beside bench.py."""
    cmd = [hipcc(), *HIPCC_FLAGS, "-o", YARDSTICK_LIB, YARDSTICK_SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    exe = [hipcc(), *[f for f in HIPCC_FLAGS if f not in ("-shared",)], "-DYS_LINK_MAIN", "-o", YARDSTICK_EXE,
           YARDSTICK_SRC]
    if verbose:
        print(" ".join(exe), flush=True)
    subprocess.run(exe, check=True)
    return YARDSTICK_LIB


def lib_is_current() -> bool:
    if not os.path.exists(LIB):
        return False
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(ROOT, "include", "mlpo.h")]
    return all(os.path.getmtime(d) <= t for d in deps)


if __name__ == "__main__":
    print(build_lib(verbose=True))
    print(build_yardsticks(verbose=True))
