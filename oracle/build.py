"""Compile the CPU oracle (test infrastructure) into oracle/libxq_oracle.so.

Strict IEEE settings: no FMA contraction, no fast-math, so that every fp32
operation in the oracle is a single correctly rounded step.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "xq_oracle.c")
LIB = os.path.join(HERE, "libxq_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build())
