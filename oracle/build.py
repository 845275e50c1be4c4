"""Compile the CPU oracle (test infrastructure) into oracle/libdam_oracle.so with gcc.

Flags matter: no fast-math and no FMA contraction, so every fp32 operation of the mask rule is
rounded on its own, as the oracle's header states.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "dam_oracle.c")
OUT = os.path.join(HERE, "libdam_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(OUT) and os.path.getmtime(OUT) >= os.path.getmtime(SRC):
        return OUT
    cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-Wall",
           "-Wextra", "-shared", "-fPIC", SRC, "-o", OUT, "-lm"]
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
