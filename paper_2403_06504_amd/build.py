"""Compile the HIP library in-tree: paper_2403_06504_amd/liblohan_adam.so (gfx950 only).

hipcc cross-compiles without a GPU.  The floating-point flags are part of the arithmetic contract:
no contraction into fused multiply-add, correctly rounded fp32 divide and square root, denormals
kept, and no packed-fp32 instruction selection.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblohan_adam.so")
SOURCES = [os.path.join(CSRC, "lohan_kernels.hip"), os.path.join(CSRC, "lohan_api.hip"),
           os.path.join(CSRC, "lohan_offload.hip"), os.path.join(CSRC, "lohan_swap_planner.hip"),
           os.path.join(CSRC, "lohan_ceiling_probe.hip")]
HEADERS = [os.path.join(CSRC, "lohan_kernels.h"), os.path.join(ROOT, "include", "lohan_adam.h"),
           os.path.join(ROOT, "include", "lohan_adam_tuning.h"),
           os.path.join(ROOT, "include", "lohan_swap_planner.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",
    "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-fno-gpu-flush-denormals-to-zero",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def build(force: bool = True, extra_flags=()) -> str:
    if not force and not stale():
        return LIB
    cmd = [HIPCC, *FLAGS, *extra_flags, "-o", LIB, *SOURCES]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True, extra_flags=sys.argv[1:]))
