"""Compiles the C part of the CPU oracle (test infrastructure) with gcc."""
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(_HERE, "liboracle_assign.so")
SRC = os.path.join(_HERE, "assign_f32.c")


def build(force: bool = False) -> str:
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", SRC, "-o", LIB, "-lm"]
        )
    return LIB


if __name__ == "__main__":
    print(build(force=True))
