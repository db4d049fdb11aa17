"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a C
driver (oracle/sanitize_check.c) calls every oracle function on buffers that end exactly where
the documented extents end; any access past them, signed overflow or invalid conversion aborts."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "sanitize_check")
    cmd = [gcc, "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-o", exe, os.path.join(ROOT, "oracle", "ngemm_oracle.c"), os.path.join(ROOT, "oracle", "sanitize_check.c"), "-lm"]
    built = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if built.returncode != 0 and "asan" in built.stdout.lower() and "cannot find" in built.stdout.lower():
        pytest.skip("no sanitizer runtime in this image: " + built.stdout[-200:])
    assert built.returncode == 0, built.stdout
    env = dict(os.environ)
    # the sanitizer runtime is linked statically; a library preloaded into every process may come first
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "4"
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout[-3000:]
    assert "sanitize_check ok" in run.stdout
