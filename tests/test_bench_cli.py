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


def test_measured_traffic_reads_a_profile_summary_only_if_taken_on_these_kernel_sources(tmp_path):
    sys.path.insert(0, ROOT)
    import bench
    name = "decode_kernel_mfma_some_workload_traffic.txt"
    body = "# rocprofv3 ... bench.py\nFETCH_BYTES_PER_LAUNCH = 1343766728\nWRITE_BYTES_PER_LAUNCH = 2130200\nMEASURED_AT_COMMIT = abc1234\n"
    (tmp_path / name).write_text(body + f"KERNEL_SOURCE_SHA = {bench.kernel_source_digest()}\n")
    t, note = bench.measured_traffic("some_workload", profiles_dir=str(tmp_path))
    assert t == 1343766728 + 2130200 and "abc1234" in note
    (tmp_path / name).write_text(body + "KERNEL_SOURCE_SHA = 0000000000000000\n")       # other sources: not this build's
    t, note = bench.measured_traffic("some_workload", profiles_dir=str(tmp_path))
    assert t is None and "other kernel sources" in note
    t, note = bench.measured_traffic("no_such_workload", profiles_dir=str(tmp_path))
    assert t is None and "no traffic summary" in note
    # the committed summaries parse (their value may be withheld if the kernels changed since)
    t, note = bench.measured_traffic("llama3_8b_decode")
    assert (t is None or 1.3e9 < t < 1.4e9) and isinstance(note, str)


def test_encode_operation_count_is_the_documented_formula():
    sys.path.insert(0, ROOT)
    import bench
    assert bench.encode_lane_ops_per_key(128) == 128 * 7 + 3 * 128 + 43 * 76
    assert bench.encode_lane_ops_per_key(64) == 64 * 6 + 3 * 64 + 22 * 76


def test_every_profile_summary_names_its_command():
    prof = os.path.join(ROOT, "profiles")
    files = [f for f in os.listdir(prof) if f.endswith((".txt", ".md"))]
    assert files
    for f in files:
        text = open(os.path.join(prof, f)).read()
        assert "rocprofv3" in text and "bench.py" in text, f
        assert os.path.getsize(os.path.join(prof, f)) < 16384, f
