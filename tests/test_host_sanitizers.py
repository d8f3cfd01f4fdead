"""The library's host-side code (tree plan, Sequoia's dynamic program, the hardware-aware choice)
under AddressSanitizer and UndefinedBehaviorSanitizer.  Only the host pass is instrumented
(the GPU has no sanitizer here), and the driver touches no GPU."""
import os
import shutil
import subprocess
import tempfile

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(ROOT, "paper_2402_12374_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def test_host_code_is_clean_under_address_and_undefined_behaviour_sanitizers():
    if not os.path.exists(HIPCC):
        pytest.skip("no hipcc")
    flags = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++20", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all",
             "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    with tempfile.TemporaryDirectory() as tmp:
        jobs = []
        for src in (os.path.join(CSRC, "tree_plan.hip"), os.path.join(CSRC, "tree_build.hip"), os.path.join(HERE, "host_sanitizer_driver.cpp")):
            obj = os.path.join(tmp, os.path.basename(src) + ".o")
            jobs.append((obj, subprocess.Popen(flags + ["-c", src, "-o", obj], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)))
        for obj, job in jobs:
            _, err = job.communicate()
            assert job.returncode == 0, err[-3000:]
        exe = os.path.join(tmp, "driver")
        link = subprocess.run([HIPCC, "--offload-arch=gfx950", "-fno-gpu-sanitize", "-fsanitize=address", "-fsanitize=undefined", "-o", exe] + [o for o, _ in jobs],
                              capture_output=True, text=True)
        assert link.returncode == 0, link.stderr[-3000:]
        run = subprocess.run([exe], capture_output=True, text=True, timeout=300,
                             env=dict(os.environ, ASAN_OPTIONS="detect_leaks=0"))
        assert run.returncode == 0 and run.stdout.strip().endswith("ok"), (run.stdout[-500:], run.stderr[-3000:])
        assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-3000:]
