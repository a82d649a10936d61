"""Host code of the library under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only, no GPU needed): the C ABI
source and the schedule / lattice-count / mask-table code are compiled with the host sanitizers (the device pass
is left as it is), linked with stand-ins for the kernel launchers and driven by tests/host_sanitize/driver.cpp over
ragged, thin, tiny and large shapes, every mask kind and the argument checks.  Any sanitizer report fails the run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2412_16112_amd", "csrc")
HERE = os.path.join(ROOT, "tests", "host_sanitize")


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not found")
def test_host_entry_points_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitize_driver")
    cmd = ["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-x", "hip",
           os.path.join(CSRC, "clear_attn_api.cpp"), os.path.join(CSRC, "schedule.cpp"),
           os.path.join(HERE, "launch_stubs.cpp"), os.path.join(HERE, "driver.cpp"), "-o", exe]
    build = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert build.returncode == 0, build.stdout[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    assert run.returncode == 0, run.stdout[-4000:]
    assert "clean under the sanitizers" in run.stdout
    assert "runtime error" not in run.stdout and "AddressSanitizer" not in run.stdout
