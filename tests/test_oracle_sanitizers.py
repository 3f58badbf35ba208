"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: oracle/*.cpp and tests/sanitizer_drive.cpp are
built with the host compiler (sanitizer runtimes linked statically) into a temporary directory and the driver runs in
a subprocess.  It takes every C entry
point of the oracle through exact-size heap buffers, truncated cards and cards with damaged headers and tables; any
out-of-bounds access, use of an uninitialised pointer, signed overflow or misaligned access ends the run with a report
and a non-zero status.  CPU only."""
import glob
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("g++") is None, reason="no host compiler")
def test_oracle_entry_points_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "sanitizer_drive")
    sources = sorted(glob.glob(os.path.join(ROOT, "oracle", "*.cpp"))) + [os.path.join(ROOT, "tests", "sanitizer_drive.cpp")]
    build = subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-ffp-contract=off",
                            "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
                            "-o", exe] + sources,
                           capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert "sanitizer drive ok" in run.stdout
