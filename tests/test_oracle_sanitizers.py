"""The oracle's C sources under AddressSanitizer and UndefinedBehaviorSanitizer.  CPU only.

A checker that reads or writes out of bounds, or leans on undefined behaviour, proves nothing:
tests/oracle_sanitize_driver.c calls every entry point of oracle/*.c on exactly-sized heap buffers
(all 65536 words through pack and unpack, a small layer with packed, unmerged and shared experts,
merge inputs with zeros / Inf / NaN, the router, the quantised codec) in a build with
-fsanitize=address,undefined; any report fails the test.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_clean_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    srcs = [os.path.join(ROOT, "tests", "oracle_sanitize_driver.c"),
            os.path.join(ROOT, "oracle", "puzzle_oracle.c"), os.path.join(ROOT, "oracle", "quant_oracle.c")]
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-static-libasan",
                           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-Wall", "-Wextra",
                           "-o", exe] + srcs + ["-lm"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="2")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    print(r.stdout, r.stderr)
    assert r.returncode == 0, r.stderr[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
    assert "oracle sanitizer drive: rc=0" in r.stdout
