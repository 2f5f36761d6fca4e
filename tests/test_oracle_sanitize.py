"""The oracle's C file under AddressSanitizer and UndefinedBehaviorSanitizer: a stand-alone driver
(oracle/sanitize_main.c) calls every entry point once on a tiny block with heap buffers of exactly the documented
sizes; any access outside a buffer or undefined arithmetic ends it with a non-zero status."""
import os
import pathlib
import shutil
import subprocess

import pytest

ROOT = pathlib.Path(__file__).resolve().parent.parent


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = tmp_path / "orc_san"
    cmd = [gcc, "-std=c11", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-ffp-contract=off", "-o", str(exe), str(ROOT / "oracle" / "sanitize_main.c"), "-lm"]
    built = subprocess.run(cmd, capture_output=True, text=True)
    if built.returncode != 0 and "sanitize" in built.stderr:
        pytest.skip("this gcc has no sanitizer runtime: " + built.stderr.strip().splitlines()[-1])
    assert built.returncode == 0, built.stderr
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert run.stdout.startswith("checksum ")
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr
