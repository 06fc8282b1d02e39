"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): ttt_oracle.c and a
small C harness are compiled with -fsanitize=address,undefined and run over packed documents with
empty and length-1 members, GQA, sampled and complete row lists, forward-only and backward calls.
Any out-of-bounds access, use after free, leak or undefined operation in the oracle fails the run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_c_is_clean_under_asan_and_ubsan(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("gcc is not installed")
    exe = tmp_path / "oracle_san"
    cmd = [gcc, "-std=c11", "-g", "-O1", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-o", str(exe),
           os.path.join(ROOT, "tests", "oracle_sanitizer_harness.c"), os.path.join(ROOT, "oracle", "ttt_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True, cwd=os.path.join(ROOT, "oracle"), capture_output=True, text=True)
    env = dict(os.environ, OMP_NUM_THREADS="3", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, f"exit {r.returncode}\nstdout:\n{r.stdout}\nstderr:\n{r.stderr[-4000:]}"
    assert "all cases passed" in r.stdout
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-4000:]
