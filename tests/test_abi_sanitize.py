"""The host side of the C ABI - validation, workspace plans, every offset between an entry point
and its launches - under AddressSanitizer and UndefinedBehaviorSanitizer, no GPU: api.hip is
built for the host with the sanitizers on, linked against stand-in launchers that check the extent
of every buffer they are handed (tests/host_sanitize/stubs.cpp), and driven through all entry
points from tiny shapes to the largest legal ones (tests/host_sanitize/driver.cpp)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

pytestmark = pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")


def test_abi_layer_under_host_sanitizers(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    src = [os.path.join(ROOT, "paper_2511_11346_amd", "csrc", "api.hip"),
           os.path.join(ROOT, "tests", "host_sanitize", "stubs.cpp"),
           os.path.join(ROOT, "tests", "host_sanitize", "driver.cpp")]
    cmd = [HIPCC, "-std=c++17", "-O1", "-g", "--offload-arch=gfx950",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2511_11346_amd", "csrc"),
           "-x", "hip", *src, "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert build.returncode == 0, build.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)          # the sanitizer runtime must come first in the library list
    run = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert "calls checked" in run.stdout and "runtime error" not in run.stderr
