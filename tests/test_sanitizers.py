"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no GPU, no GPU sanitizer): the oracle's C
file with a driver that runs every entry point, and the library's host side (plans, codebooks, argument checks,
dispatch) with stubbed kernel launchers.  The drivers live in tests/sanitize/."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1",
           OMP_NUM_THREADS="4")


def _run(cmd, **kw):
    return subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not found")
def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    res = _run(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                "-fno-omit-frame-pointer", "-fopenmp", os.path.join(SAN, "oracle_driver.c"), "-o", exe, "-lm"])
    assert res.returncode == 0, res.stderr
    res = _run([exe], env=ENV)
    assert res.returncode == 0 and "oracle driver ok" in res.stdout, res.stdout + res.stderr


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", shutil.which("hipcc")):
        if cand and os.path.exists(cand):
            return cand
    return None


@pytest.mark.skipif(_hipcc() is None, reason="hipcc not found")
def test_library_host_side_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "host_san")
    csrc = os.path.join(ROOT, "paper_2605_21226_amd", "csrc")
    # host pass only under the sanitizers (each -fsanitize= directly after -Xarch_host); the device pass is untouched
    res = _run([_hipcc(), "-O1", "-g", "-std=c++17", "--offload-arch=gfx950", "-x", "hip",
                "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
                "-I" + os.path.join(ROOT, "include"), "-I" + csrc, "-Wno-unused-command-line-argument",
                os.path.join(csrc, "octopus_host.cpp"), os.path.join(SAN, "host_driver.cpp"), "-o", exe,
                "-fsanitize=address", "-fsanitize=undefined"])
    assert res.returncode == 0, res.stderr[-4000:]
    # (leak detection off here: the HIP runtime this executable links keeps its own allocations until exit)
    res = _run([exe], env=dict(ENV, ASAN_OPTIONS="detect_leaks=0"))
    assert res.returncode == 0 and "host driver ok" in res.stdout, res.stdout + res.stderr[-4000:]
