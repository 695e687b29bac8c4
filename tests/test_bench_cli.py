"""bench.py's host-side argument handling (no GPU needed)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args, env=None):
    e = dict(os.environ)
    e.update(env or {})
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args],
                          capture_output=True, text=True, env=e, timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""
    # launched under a multi-rank launcher: the same refusal
    r = _run(env={"WORLD_SIZE": "4"})
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_unknown_workload_is_an_error():
    r = _run("--workload", "no_such_workload")
    assert r.returncode != 0
