"""The runtime's host side (index build over several builders, pooled buffers, queue and condition variables, the
sampler) built without device code under ThreadSanitizer and AddressSanitizer and driven by a stress program
(tests/sanitize/host_stress.cpp): many builds in flight from two calling threads, views read and graphs released
while others are being built.  CPU only (host-only contexts, device < 0)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2408_08490_amd", "csrc")
SAN = os.path.join(ROOT, "tests", "sanitize")


@pytest.mark.parametrize("sanitizer", ["thread", "address"])
def test_host_runtime_under_sanitizer(sanitizer, tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path / ("host_stress_" + sanitizer))
    srcs = [os.path.join(CSRC, f) for f in ("api.cpp", "host_build.cpp", "sampler.cpp")] + \
           [os.path.join(SAN, f) for f in ("launch_stubs.cpp", "host_stress.cpp")]
    cmd = [gxx, "-std=c++20", "-O1", "-g", "-fsanitize=" + sanitizer, "-fno-omit-frame-pointer", "-D__HIP_PLATFORM_AMD__",
           "-I/opt/rocm/include", "-w", "-o", exe] + srcs + ["-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-lpthread"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-4000:]
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=0 exitcode=66", ASAN_OPTIONS="detect_leaks=0 exitcode=66")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    report = (run.stdout + run.stderr)[-6000:]
    assert run.returncode == 0 and "host stress ok" in run.stdout, report
    assert "WARNING: ThreadSanitizer" not in report and "ERROR: AddressSanitizer" not in report, report
