"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer: the planner and the C ABI are compiled
(without the GPU code, which is stubbed) together with a driver that plans every benchmark workload and a set
of awkward ones, walks boxes, tiles and manifests, and exercises the error paths."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2312_05181_amd", "csrc")
NATIVE = os.path.join(ROOT, "tests", "native")


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_planner_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "plan_driver")
    srcs = [os.path.join(CSRC, f) for f in ("layout.cpp", "planner.cpp", "dataset.cpp", "api.cpp")]
    srcs += [os.path.join(NATIVE, "hip_stubs.cpp"), os.path.join(NATIVE, "plan_driver.cpp")]
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-static-libasan", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", exe] + srcs
    subprocess.run(cmd, check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]
    assert "all checks passed" in res.stdout
