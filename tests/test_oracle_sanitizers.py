"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only):
oracle/sanitize_driver.c is compiled together with the oracle's source, in both precisions,
and run as a program of its own; any finding ends it with a non-zero status."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("real", ["double", "float"])
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path, real):
    exe = str(tmp_path / f"sanitize_{real}")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fno-omit-frame-pointer",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", f"-DREAL={real}",
           "-o", exe, os.path.join(ROOT, "oracle", "sanitize_driver.c"), "-lm"]
    subprocess.run(cmd, check=True, cwd=os.path.join(ROOT, "oracle"))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    out = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-4000:]
    assert "status 0" in out.stdout
