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


def test_counter_traffic_is_reported_only_for_unchanged_kernel_sources(tmp_path, monkeypatch):
    import json
    sys.path.insert(0, ROOT)
    import bench
    h = bench.source_hash("apply_kernel")
    assert len(h) == 16 and h == bench.source_hash("apply_kernel")
    rec = {"workload": "gpt2_small", "n": 10, "m": 2, "storage": "f32", "kernel": "apply_kernel",
           "fetched_bytes": 100, "written_bytes": 20, "source_sha16": h}
    f = tmp_path / "t.txt"
    f.write_text(json.dumps({"records": [rec]}))
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(f))
    assert bench.measured_traffic("gpt2_small", 10, 2, "f32", "apply_kernel") == 120
    assert bench.measured_traffic("gpt2_small", 11, 2, "f32", "apply_kernel") is None
    rec["source_sha16"] = "0" * 16            # the kernel has changed since the counters were taken
    f.write_text(json.dumps({"records": [rec]}))
    assert bench.measured_traffic("gpt2_small", 10, 2, "f32", "apply_kernel") is None
    monkeypatch.setattr(bench, "TRAFFIC_FILE", str(tmp_path / "missing.txt"))
    assert bench.measured_traffic("gpt2_small", 10, 2, "f32", "apply_kernel") is None
