"""Compile the CPU oracle (plain C, gcc) into oracle/libqn_oracle.so.

Test infrastructure only: the product library never links or loads this.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libqn_oracle.so")
LIB_SANITIZED = os.path.join(HERE, "libqn_oracle_san.so")


def build(verbose: bool = False) -> str:
    # -O2 without -ffast-math: the summation order written in the source is
    # the summation order that runs.
    cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, os.path.join(HERE, "qn_oracle.c"), "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


def build_sanitized(verbose: bool = False) -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (host
    code only), for the test that runs the pin suite on it.  A process that loads
    it must have the AddressSanitizer runtime preloaded (asan_runtime())."""
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer", "-o", LIB_SANITIZED,
           os.path.join(HERE, "qn_oracle.c"), "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB_SANITIZED


def asan_runtime() -> str:
    """Path of gcc's AddressSanitizer runtime library."""
    return subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()


if __name__ == "__main__":
    print(build(verbose=True))
