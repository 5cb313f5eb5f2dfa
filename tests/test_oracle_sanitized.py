"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer: a driver
(tests/c/oracle_sanitizer_driver.c) calls every function on small odd-sized inputs in exactly
sized heap blocks; any out-of-bounds access, use after free, signed overflow or misaligned
access aborts it."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_c_code_is_clean_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-o", exe, os.path.join(ROOT, "tests", "c", "oracle_sanitizer_driver.c"),
           os.path.join(ROOT, "oracle", "oracle.c"), "-lm"]
    subprocess.check_call(cmd)
    # (the link-order check is off because the environment may preload a library of its own)
    env = dict(os.environ, OMP_NUM_THREADS="3", ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stderr[-2000:]
    assert "checksum" in run.stdout and "ERROR" not in run.stderr
