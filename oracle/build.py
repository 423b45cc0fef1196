"""Compiles the C part of the oracle with gcc (test infrastructure only)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "cleave_oracle.c")
LIB = os.path.join(HERE, "libcleave_oracle.so")

# -O2 and nothing that reorders floating point: no -ffast-math, no FMA
# contraction (an fp64 FMA would only make the reference more accurate, but
# the fp32 fold must be plain IEEE adds).
FLAGS = ["-O2", "-fopenmp", "-ffp-contract=off", "-shared", "-fPIC", "-std=c11", "-Wall"]


def build(force=False):
    stale = (not os.path.exists(LIB)) or os.path.getmtime(LIB) < os.path.getmtime(SRC)
    if force or stale:
        subprocess.check_call(["gcc"] + FLAGS + ["-o", LIB, SRC])
    return LIB


if __name__ == "__main__":
    print(build(force=True))
