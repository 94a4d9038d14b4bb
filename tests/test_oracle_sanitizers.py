"""AddressSanitizer + UndefinedBehaviorSanitizer pass over the C oracle (CPU only).

oracle/sanitize_check.c includes the oracle's source and drives every exported routine over small seeded inputs
(ragged lengths, both tile orders, the study formats, chunked prefill, decode with a partly filled last block).
The sanitizers abort on the first finding, so a zero exit status means a clean pass."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "oracle_sanitize_check")
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fno-fast-math", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           os.path.join(ROOT, "oracle", "sanitize_check.c"), "-o", exe, "-lm"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and ("asan" in built.stderr or "ubsan" in built.stderr):
        pytest.skip("this gcc has no sanitizer runtime: " + built.stderr.strip().splitlines()[-1])
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, OMP_NUM_THREADS="8", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert "oracle sanitizer pass: ok" in run.stdout
