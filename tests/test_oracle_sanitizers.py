"""The CPU checker's C code under AddressSanitizer and UndefinedBehaviorSanitizer: a driver
(oracle_sanitizer_driver.c) calls every entry point on small inputs with the edge cases the
parity tests rely on; any report from either sanitizer fails the test."""
import os
import shutil
import subprocess
import tempfile

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE = os.path.join(os.path.dirname(HERE), "oracle")
SOURCES = ["tree_attn_oracle.c", "verify_oracle.c", "draft_sample_oracle.c", "verify_baselines_oracle.c"]


def test_checker_is_clean_under_address_and_undefined_behaviour_sanitizers():
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "driver")
        cmd = ["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-static-libasan", "-fno-sanitize-recover=all",
               "-fno-omit-frame-pointer", "-o", exe, os.path.join(HERE, "oracle_sanitizer_driver.c")]
        cmd += [os.path.join(ORACLE, s) for s in SOURCES] + ["-lm"]
        built = subprocess.run(cmd, capture_output=True, text=True)
        if built.returncode != 0 and "sanitize" in built.stderr and "cannot find" in built.stderr:
            pytest.skip("sanitizer runtime not installed")
        assert built.returncode == 0, built.stderr
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
        run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
        assert run.returncode == 0 and run.stdout.strip() == "ok", (run.stdout, run.stderr[-2000:])
        assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-2000:]
