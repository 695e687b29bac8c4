"""Compile the CPU oracle (plain C, gcc) into oracle/libqn_oracle.so.

Test infrastructure only: the product library never links or loads this.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libqn_oracle.so")


def build(verbose: bool = False) -> str:
    # -O2 without -ffast-math: the summation order written in the source is
    # the summation order that runs.
    cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, os.path.join(HERE, "qn_oracle.c"), "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
