"""Compile the CPU oracle (plain C + OpenMP) into oracle/liblpg_oracle.so.

Test infrastructure only: nothing in the product package imports this.
Portable flags only (no -march=native): the library is built on one machine
and run on another.  -ffp-contract=off keeps every multiply and add separate,
so the sums are the ones the source spells out.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "lpg_oracle.c")
LIB = os.path.join(HERE, "liblpg_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-ftree-vectorize", "-ffp-contract=off", "-fopenmp", "-fPIC",
           "-shared", "-std=c11", "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build())
