"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only).

oracle/sanitize_check.c includes oracle.c and calls every entry point on small inputs in
buffers of exactly the documented sizes; this test compiles it with gcc's sanitizers, once
without and once with OpenMP, and runs it.  Any read or write past the end of a buffer, use
after free, signed overflow or bad shift in the oracle ends the run with a report."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "sanitize_check.c")


@pytest.mark.parametrize("openmp", [False, True], ids=["serial", "openmp"])
def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path, openmp):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "sanitize_check")
    cmd = [gcc, "-O1", "-g", "-ffp-contract=off", "-mfma", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", SRC, "-lm", "-o", exe]
    if openmp:
        cmd.insert(1, "-fopenmp")
    built = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if built.returncode != 0 and "sanitize" in built.stdout and "cannot find" in built.stdout:
        pytest.skip("this gcc has no sanitizer runtime: " + built.stdout[-200:])
    assert built.returncode == 0, built.stdout[-2000:]
    env = dict(os.environ)
    # (a library preloaded by the environment may come before the sanitizer's runtime)
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "4"
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env,
                         timeout=300)
    assert run.returncode == 0 and "sanitize_check: ok" in run.stdout, run.stdout[-3000:]
