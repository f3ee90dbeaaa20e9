"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

tests/oracle_sanitize_driver.c calls every exported function of oracle/tri_oracle.c on heap buffers of exactly the
contracted sizes; both files are compiled here with gcc -fsanitize=address,undefined (the sanitizer runtime linked
statically, so nothing has to be preloaded) and the driver must finish without a report."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "oracle_sanitize")
    cmd = [gcc, "-O1", "-g", "-std=c11", "-Wall", "-Wextra", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", os.path.join(ROOT, "oracle", "tri_oracle.c"),
           os.path.join(ROOT, "tests", "oracle_sanitize_driver.c"), "-lm", "-o", exe]
    built = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if built.returncode != 0 and "asan" in built.stdout.lower() and "cannot find" in built.stdout.lower():
        pytest.skip("this gcc has no static sanitizer runtime")
    assert built.returncode == 0, built.stdout
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout
    assert "all checks passed" in run.stdout
