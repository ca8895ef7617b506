"""Compiles the C oracle into oracle/librocket_oracle.so (gcc, OpenMP).

TEST INFRASTRUCTURE ONLY: part of the CPU oracle."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "rocket_oracle.c")
LIB = os.path.join(HERE, "librocket_oracle.so")


def build(force=True):
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
