"""CPU-side safety nets: the oracle's pin suite under AddressSanitizer and
UndefinedBehaviorSanitizer, and the library's launch arithmetic (grids, tile
counts, slab lengths, workspace sizes) checked by a host build of the same header
the launchers use, also under the sanitizers."""
import os
import subprocess
import sys

import pytest

from oracle import build as oracle_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN_FLAGS = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
             "-fno-omit-frame-pointer", "-g", "-O1"]


def _env(lib):
    env = dict(os.environ)
    env.update(QN_ORACLE_LIB=lib, LD_PRELOAD=oracle_build.asan_runtime(),
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:exitcode=23")
    return env


def test_oracle_pins_pass_under_address_and_ub_sanitizers():
    lib = oracle_build.build_sanitized()
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")],
                       env=_env(lib), capture_output=True, text=True, cwd=ROOT, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    assert " passed" in r.stdout and "failed" not in r.stdout


def test_the_sanitized_build_catches_a_planted_overrun(tmp_path):
    # the net itself: a copy of the oracle whose row-mean loop reads one worker too
    # many must be caught (the mistake is planted in the copy, on the CPU)
    src = open(os.path.join(ROOT, "oracle", "qn_oracle.c")).read()
    good = "        for (int k = 0; k < m; ++k)\n            s += elem(X, dtype, (int64_t)k * ld + i);"
    assert src.count(good) == 1
    bad = good.replace("k < m", "k <= m")
    (tmp_path / "qn_oracle.c").write_text(src.replace(good, bad))
    (tmp_path / "qn_oracle.h").write_text(open(os.path.join(ROOT, "oracle", "qn_oracle.h")).read())
    lib = str(tmp_path / "libbad.so")
    subprocess.check_call(["gcc", "-std=c99", "-fPIC", "-shared", *SAN_FLAGS, "-o", lib,
                           str(tmp_path / "qn_oracle.c"), "-lm"])
    code = ("import numpy as np, oracle\n"
            "x = np.ones((4, 64), np.float32)\n"
            "print(oracle.row_means(x)[0])\n")
    r = subprocess.run([sys.executable, "-c", code], env=_env(lib), capture_output=True,
                       text=True, cwd=ROOT, timeout=120)
    assert r.returncode != 0 and "AddressSanitizer" in r.stderr


def test_launch_arithmetic_on_the_host(tmp_path):
    exe = str(tmp_path / "launch_math_check")
    subprocess.check_call(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", *SAN_FLAGS,
                           "-I", os.path.join(ROOT, "include"),
                           "-I", os.path.join(ROOT, "paper_1709_05069_amd", "csrc"),
                           os.path.join(ROOT, "tests", "host", "launch_math_check.cpp"),
                           "-o", exe])
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "launch arithmetic ok" in r.stdout
