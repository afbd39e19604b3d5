"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a small C
driver calls every oracle entry point on exactly-sized heap arrays; any out-of-bounds index, misaligned
access or undefined arithmetic in oracle/pa_oracle.c aborts the run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / "oracle_sanitized")
    # the sanitizer runtime is linked statically so that it needs no place in the preload order
    cmd = [gcc, "-std=c99", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
           os.path.join(ROOT, "oracle", "pa_oracle.c"), os.path.join(ROOT, "oracle", "sanitize_driver.c"),
           "-o", exe, "-lm"]
    built = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if built.returncode != 0 and ("cannot find" in built.stdout or "libasan" in built.stdout):
        pytest.skip("no static sanitizer runtime in this toolchain: " + built.stdout[-200:])
    assert built.returncode == 0, built.stdout
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout
    assert run.stdout.strip().endswith("ok"), run.stdout
