"""The C oracle under AddressSanitizer + UndefinedBehaviorSanitizer, on the CPU.

tests/c_abi/oracle_sanitize.c calls every entry point of oracle/seer_oracle.c on exactly-sized heap
buffers (three selection modes, contiguous and paged caches, an empty sequence, a partial last block,
several new tokens, both front-end projections, the training-side ground truth); the build below aborts
on the first out-of-bounds access or undefined operation.
"""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-static-libasan",
           os.path.join(HERE, "c_abi", "oracle_sanitize.c"), os.path.join(ROOT, "oracle", "seer_oracle.c"),
           "-fopenmp", "-lm", "-o", exe]
    b = subprocess.run(cmd, capture_output=True, text=True)
    assert b.returncode == 0, b.stderr
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, f"exit {r.returncode}\n{r.stdout}\n{r.stderr}"
    assert "oracle sanitizer run clean" in r.stdout
