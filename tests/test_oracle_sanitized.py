"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only; no GPU involved).

tests/oracle_selftest.c drives every oracle function on seeded random shapes with exact-size heap buffers, so an
out-of-bounds access or undefined arithmetic inside the oracle fails here even when its results happen to be right."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE = os.path.join(ROOT, "oracle")


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "oracle_selftest"
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-Wall", "-Wextra", "-Werror", "-pthread", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", f"-I{ORACLE}", os.path.join(ROOT, "tests", "oracle_selftest.c"),
           os.path.join(ORACLE, "tutti_oracle.c"), "-o", str(exe)]
    build = subprocess.run(cmd, capture_output=True, text=True)
    if build.returncode != 0 and "asan" in build.stderr.lower() and "cannot find" in build.stderr.lower():
        pytest.skip("no static sanitizer runtime on this machine")
    assert build.returncode == 0, build.stderr[-2000:]
    run = subprocess.run([str(exe), "400"], capture_output=True, text=True, timeout=600)
    assert run.returncode == 0, (run.stdout[-500:], run.stderr[-3000:])
    assert run.stdout.strip() == "ok 400"
