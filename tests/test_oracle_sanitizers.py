"""Host-side sanitizer run of the CPU oracle (AddressSanitizer + UndefinedBehaviorSanitizer):
oracle/hq_oracle.c is compiled together with a small C driver that calls every one of its
functions on small ragged inputs, and the binary must run to the end without a report.  CPU only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    build = subprocess.run(
        ["gcc", "-std=c11", "-O1", "-g", "-fno-omit-frame-pointer", "-fopenmp",
         "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
         os.path.join(ROOT, "tests", "oracle_sanitize_driver.c"), os.path.join(ROOT, "oracle", "hq_oracle.c"),
         "-lm", "-o", exe],
        stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert build.returncode == 0, build.stdout
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout[-4000:]
    assert "oracle sanitizer driver: ok" in run.stdout
    assert "runtime error" not in run.stdout and "AddressSanitizer" not in run.stdout, run.stdout[-4000:]
