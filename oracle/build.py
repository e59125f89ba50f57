"""Compile the CPU oracle (plain C) into oracle/libaa_ref.so with gcc.

Test infrastructure: building the checker is not using it.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libaa_ref.so")


def build(force: bool = True) -> str:
    src = os.path.join(HERE, "aa_ref.c")
    hdr = os.path.join(HERE, "aa_ref.h")
    if not force and os.path.exists(LIB):
        if os.path.getmtime(LIB) >= max(os.path.getmtime(src), os.path.getmtime(hdr)):
            return LIB
    cmd = ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wextra", "-o", LIB, src, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
