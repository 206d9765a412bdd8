"""The C-ABI front end (argument validation, workspace sizing, the split-of-K heuristics) built for the HOST with
AddressSanitizer and UndefinedBehaviorSanitizer, kernel launchers replaced by stubs, and driven through every entry
point's error paths by tests/host_sanitizer/driver.cpp.  No GPU involved: sanitizers run on host code only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "host_sanitizer")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_validation_under_address_and_undefined_behavior_sanitizers(tmp_path):
    exe = str(tmp_path / "abi_sanitizer_driver")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           os.path.join(ROOT, "paper_2505_14638_amd", "csrc", "api.hip"),
           os.path.join(HERE, "launch_stubs.cpp"), os.path.join(HERE, "driver.cpp"), "-o", exe]
    build = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    assert build.returncode == 0, build.stdout[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0")        # the HIP runtime's own start-up allocations are not ours
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120, env=env)
    assert run.returncode == 0 and "all checks passed" in run.stdout, run.stdout[-4000:]
    shutil.rmtree(tmp_path, ignore_errors=True)
