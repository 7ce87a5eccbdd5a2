"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU).

The oracle is plain C with hand-indexed buffers and OpenMP regions; this builds it with gcc's sanitizers together
with a small driver that calls every batch driver and the entry points with (m, s) given, and expects a clean exit.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-o", exe,
           os.path.join(ROOT, "tests", "oracle_sanitize_driver.c"), os.path.join(ROOT, "oracle", "expm_oracle.c"), "-lm"]
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and "asan" in (build.stderr or "").lower() and "cannot find" in build.stderr.lower():
        pytest.skip("the sanitizer runtime libraries are not installed")
    assert build.returncode == 0, build.stderr
    env = dict(os.environ)
    # libraries preloaded into every process of this machine may come before the sanitizer runtime: do not insist
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "3"
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, (run.returncode, run.stdout[-2000:], run.stderr[-4000:])
    assert "checksum" in run.stdout and "runtime error" not in run.stderr and "ERROR: AddressSanitizer" not in run.stderr
