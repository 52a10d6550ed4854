"""Host-side behaviour of bench.py that needs no GPU."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    res = _run("--gpus", "2")
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_measured_traffic_reads_the_committed_profile_summary():
    sys.path.insert(0, ROOT)
    import bench
    t = bench.measured_traffic("llama3_8b_decode")
    assert isinstance(t, int) and 1.3e9 < t < 1.4e9          # FETCH + WRITE bytes per launch from profiles/
    assert bench.measured_traffic("no_such_workload") is None


def test_every_profile_summary_names_its_command():
    prof = os.path.join(ROOT, "profiles")
    files = [f for f in os.listdir(prof) if f.endswith((".txt", ".md"))]
    assert files
    for f in files:
        text = open(os.path.join(prof, f)).read()
        assert "rocprofv3" in text and "bench.py" in text, f
        assert os.path.getsize(os.path.join(prof, f)) < 16384, f
