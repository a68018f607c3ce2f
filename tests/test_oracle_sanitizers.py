"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): oracle/sanitize_check.c
calls every oracle function on small awkward inputs with exactly-sized buffers; any out-of-bounds access,
signed overflow or invalid shift aborts the program."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE = os.path.join(ROOT, "oracle")


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "orc_san")
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-ffp-contract=off", "-D_DEFAULT_SOURCE",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-fno-omit-frame-pointer",
           "-Wall", "-Wextra", "-Werror", "-o", exe,
           os.path.join(ORACLE, "sanitize_check.c"), os.path.join(ORACLE, "sbits_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True, cwd=ORACLE)
    r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "oracle sanitize check: ok" in r.stdout
    assert "ERROR" not in r.stdout and "runtime error" not in r.stdout
