"""The host planners (partition, micro-group plan, TP schedule) run under
AddressSanitizer and UBSan on random inputs, with output arrays of exactly the documented
sizes.  CPU only; device code is not part of this build."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2602_06079_amd", "csrc")
HOST = ["error.cpp", "partition.cpp", "microgroup.cpp", "tp_schedule.cpp"]


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_planners_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-ffp-contract=off", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(ROOT, "tests", "host_sanitize_driver.cpp")] + [os.path.join(CSRC, f) for f in HOST] + ["-o", exe]
    build = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if build.returncode != 0 and "cannot find" in build.stdout:
        pytest.skip("sanitizer runtimes not installed: " + build.stdout[-200:])
    assert build.returncode == 0, build.stdout
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=300)
    assert run.returncode == 0 and run.stdout.strip().endswith("ok"), run.stdout[-2000:]
