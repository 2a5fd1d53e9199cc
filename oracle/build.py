"""Compile the CPU oracle (plain C) into oracle/liboracle.so.

Test infrastructure: the oracle is the checker, not the product.  Flags keep
the arithmetic plain: -O2, no fast-math, no FMA contraction.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = ["dpc_oracle.c", "dpc_brute.c", "dpc_ext_oracle.c", "dpc_ext_brute.c",
           "dpc_sweep_oracle.c"]
LIB = os.path.join(HERE, "liboracle.so")


def build(force: bool = True) -> str:
    srcs = [os.path.join(HERE, s) for s in SOURCES]
    if not force and os.path.exists(LIB):
        if all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in srcs):
            return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
           "-fno-fast-math", "-Wall", "-Wextra", "-o", LIB] + srcs + ["-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
