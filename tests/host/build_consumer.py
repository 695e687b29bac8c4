"""Builds tests/host/abi_consumer (a plain-C user of libqn's ABI, with the CPU
oracle linked in as its checker) with gcc against the HIP runtime.  Test infrastructure only."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
EXE = os.path.join(HERE, "abi_consumer")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def sources():
    return [os.path.join(HERE, "abi_consumer.c"), os.path.join(ROOT, "oracle", "qn_oracle.c"),
            os.path.join(ROOT, "oracle", "qn_oracle.h"), os.path.join(ROOT, "include", "qn.h")]


def stale() -> bool:
    """True when the executable is missing or older than what it is built from."""
    if not os.path.exists(EXE):
        return True
    built = os.path.getmtime(EXE)
    return any(os.path.getmtime(s) > built for s in sources())


def build(verbose: bool = False) -> str:
    pkg = os.path.join(ROOT, "paper_1709_05069_amd")
    cmd = ["gcc", "-std=c99", "-O2", "-Wall", "-Wno-maybe-uninitialized", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "oracle"),
           "-I", os.path.join(ROCM, "include"),
           os.path.join(HERE, "abi_consumer.c"), os.path.join(ROOT, "oracle", "qn_oracle.c"),
           "-L", pkg, "-lqn", "-L", os.path.join(ROCM, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../../paper_1709_05069_amd", "-Wl,-rpath," + os.path.join(ROCM, "lib"), "-lm", "-o", EXE]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return EXE


if __name__ == "__main__":
    print(build(verbose=True))
