"""The CPU oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer (host only, no GPU): a small driver
(tests/sanitize/oracle_sanitize.c) is compiled together with oracle/salr_oracle.c and walks every oracle entry point
over ragged shapes with exactly-sized heap buffers; any out-of-bounds access or undefined arithmetic ends it with a
non-zero status."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_oracle_clean_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
           "-fno-omit-frame-pointer", "-Wall", "-Wextra", "-o", exe,
           os.path.join(ROOT, "tests", "sanitize", "oracle_sanitize.c"), os.path.join(ROOT, "oracle", "salr_oracle.c")]
    build = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert build.returncode == 0, build.stdout
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout[-4000:]
    assert "shapes clean" in run.stdout
