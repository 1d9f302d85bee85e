"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: oracle/sb_oracle.c is
built with a small C driver (oracle/sanitize_driver.c) into a stand-alone executable, so no
sanitizer runtime has to be preloaded into Python, and run on tiny shapes: full rows, a row
range, an empty range, T = 1, with and without the remainder bias, forward and backward, the
dense weights, and the error paths.  A clean exit is the assertion."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-omit-frame-pointer",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-Wall", "-Wextra",
           "-o", exe, os.path.join(ROOT, "oracle", "sanitize_driver.c"),
           os.path.join(ROOT, "oracle", "sb_oracle.c"), "-lm"]
    built = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert built.returncode == 0, built.stdout
    env = dict(os.environ)
    # whatever the environment preloads stays as it is: the link-order check is relaxed instead
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "4"
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout
    assert "oracle sanitizer run clean" in run.stdout
    assert "runtime error" not in run.stdout and "AddressSanitizer" not in run.stdout, run.stdout
