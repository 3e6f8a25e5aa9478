"""Host-side checks of the benchmark script's contract (no GPU needed)."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT,
                          stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2")
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_stored_traffic_records_are_consistent_and_expire_with_the_sources():
    """The roofline's `traffic` figures are only reported while the kernel and planner
    sources hash to what the counters were taken on (null otherwise); the committed records
    carry the copy-calibrated scales and add up."""
    sys.path.insert(0, ROOT)
    import bench
    for kernel in sorted(bench.TRAFFIC_SOURCES):
        path, digest = bench._traffic_file(kernel, "c5_stress")
        rec = json.load(open(path))
        assert rec["fetch_scale"] == 2.0 and rec["write_scale"] == 1.0
        want = (rec["fetch_size_kib_per_launch"] * 2.0 + rec["write_size_kib_per_launch"]) * 1024
        assert abs(rec["hbm_bytes_per_launch"] - want) <= 1.0
        got = bench.measured_traffic("c5_stress", kernel)
        if rec["source_sha256_16"] == digest:
            assert got == rec["hbm_bytes_per_launch"]
        else:
            assert got is None          # counters predate the sources: not reported
    assert bench.measured_traffic("no_such_workload") is None
