"""The C ABI used from plain C: tests/host/abi_consumer.c allocates with hipMalloc,
calls qn_update, qn_update_ws and qn_update_noalloc with raw device pointers on a
stream of its own, and checks each against the CPU oracle linked into it.  No
Python object crosses the boundary; this test only starts the program."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, os.path.join(ROOT, "tests", "host"))
import build_consumer  # noqa: E402


def test_consumer_compiles_and_links_against_the_public_header():
    exe = build_consumer.build()
    out = subprocess.run(["ldd", exe], capture_output=True, text=True).stdout
    assert "libqn.so" in out and "not found" not in out.split("libqn.so")[1].splitlines()[0]


@pytest.mark.gpu
def test_plain_c_consumer_matches_the_oracle():
    exe = build_consumer.build() if build_consumer.stale() else build_consumer.EXE
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    print(r.stdout)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "C consumer: all ok" in r.stdout
    assert r.stdout.count("bit-identical -> ok") == 4
