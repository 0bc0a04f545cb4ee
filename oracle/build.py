"""Compile the C oracle into oracle/liblohan_oracle.so with the host compiler.

Test infrastructure only.  The flags matter for what the oracle means: no fused multiply-add
(-ffp-contract=off), no value-changing optimisation (-fno-fast-math), plain x86-64 SSE arithmetic.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "lohan_oracle.c")
LIB = os.path.join(HERE, "liblohan_oracle.so")

CFLAGS = ["-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC", "-shared",
          "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    """Build the shared object; with force=False an up-to-date one is kept."""
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", *CFLAGS, "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
