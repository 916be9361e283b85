"""Compile the CPU oracle (test infrastructure) into oracle/libfq_oracle.so.

-ffp-contract=off keeps every floating-point operation of the oracle a single
IEEE binary32 operation (the fused multiply-adds it uses are written as fmaf).
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "fq_oracle.c")
LIB = os.path.join(HERE, "libfq_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
