"""Compile the CPU oracle (test infrastructure) into oracle/libdam_oracle.so with gcc.

Flags matter: no fast-math and no FMA contraction, so every fp32 operation of the mask rule is
rounded on its own, as the oracle's header states.

build(sanitize=True) makes a second library, oracle/libdam_oracle_asan.so, with AddressSanitizer and
UndefinedBehaviorSanitizer (host code only); the oracle package loads it when DAM_ORACLE_SANITIZE=1 is
set, and tests/test_oracle_sanitized.py runs the oracle's own tests over it.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "dam_oracle.c")
OUT = os.path.join(HERE, "libdam_oracle.so")
OUT_ASAN = os.path.join(HERE, "libdam_oracle_asan.so")


def build(force: bool = True, sanitize: bool = False) -> str:
    out = OUT_ASAN if sanitize else OUT
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
        return out
    cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-Wall",
           "-Wextra", "-shared", "-fPIC"]
    if sanitize:
        cmd += ["-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
    subprocess.run(cmd + [SRC, "-o", out, "-lm"], check=True)
    return out


def asan_runtime() -> str:
    """Path of gcc's libasan.so, to be preloaded into an uninstrumented python."""
    return subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True).stdout.strip()


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv, sanitize="--sanitize" in sys.argv))
