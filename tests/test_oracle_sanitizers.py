"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): a small C program
(tests/oracle_sanitize_main.c) compiled together with oracle/lcn_oracle.c walks every exported
routine through ragged little problems; any report, leak or non-zero status fails the test."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not found")
def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    src = os.path.join(ROOT, "tests", "oracle_sanitize_main.c")
    # the oracle's own flags (no contraction, OpenMP) plus the sanitizers; the runtime is linked
    # statically so that it does not depend on the order of preloaded libraries
    cmd = ["gcc", "-O1", "-g", "-ffp-contract=off", "-fopenmp", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-o", exe, src, "-lm"]
    subprocess.check_call(cmd)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    res = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert res.returncode == 0, res.stdout[-4000:]
    assert "runtime error" not in res.stdout and "AddressSanitizer" not in res.stdout, res.stdout[-4000:]
    assert "oracle sanitizer run: rc=0" in res.stdout
