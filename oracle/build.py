"""Compile the C oracle into oracle/libmolora_oracle.so (gcc, OpenMP, no fast-math)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRCS = [os.path.join(HERE, "molora_oracle.c"), os.path.join(HERE, "molora_oracle_mix.c")]
LIB = os.path.join(HERE, "libmolora_oracle.so")

# -ffp-contract=off / no fast-math: the loops' written summation order is the order run.
# x86-64-v3 (AVX2) keeps the binary runnable on hosts without AVX-512.
CFLAGS = ["-O3", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
          "-fno-fast-math", "-march=x86-64-v3", "-Wall", "-Wextra"]


def build(force=True):
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(f) for f in SRCS):
        return LIB
    cmd = ["gcc", *CFLAGS, *SRCS, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
    sys.exit(0)
