"""Compile the CPU oracle (plain C, OpenMP) into oracle/libpass_oracle.so."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "pass_oracle.c")
LIB = os.path.join(HERE, "libpass_oracle.so")


def build(force: bool = False) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    # -ffp-contract=off: a product and a sum stay two roundings (no fused multiply-add), so the vector
    # code -O3 -mavx2 makes of the inner loops gives the bits the scalar code gives
    cmd = ["gcc", "-std=c11", "-O3", "-mavx2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
