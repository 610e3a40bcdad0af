"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only).

oracle/sanitize_main.c calls every C function of the oracle on exact-size heap buffers with ragged
shapes; the program is built with the sanitizers linked statically and run as a child process."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-ffp-contract=off", "-Wall", "-Wextra",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
           "-I", os.path.join(ROOT, "oracle"), "-o", exe, os.path.join(ROOT, "oracle", "sanitize_main.c"), "-lm"]
    built = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    if built.returncode != 0 and b"cannot find" in built.stdout:
        pytest.skip("static sanitizer runtimes are not installed: " + built.stdout.decode()[-200:])
    assert built.returncode == 0, built.stdout.decode()
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.PIPE, env=env, timeout=300)
    out, err = run.stdout.decode(), run.stderr.decode()
    assert run.returncode == 0, err[-2000:]
    assert out.strip().endswith("ok"), out
    assert "AddressSanitizer" not in err and "runtime error" not in err, err[-2000:]
