"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a small driver
calls every entry point over modes, bit widths, both formats, odd lengths and short last groups; any
out-of-bounds access or undefined arithmetic in the oracle ends it with a report."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-ffp-contract=off", "-fno-fast-math", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-Wall", "-Werror", "-I", os.path.join(ROOT, "oracle"),
           os.path.join(ROOT, "oracle", "adacc_oracle.c"), os.path.join(ROOT, "tests", "csrc", "oracle_sanitize_main.c"),
           "-lm", "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", LD_PRELOAD="")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr
    assert "rc=0" in run.stdout
