"""The host runtime (zz_api.cpp, zz_transport.cpp) under AddressSanitizer and
UndefinedBehaviorSanitizer, driven by tests/host_runtime_sanitized.cpp: thousands of
append / prefill / decode calls at equal and unequal lengths with recorders in place of the
kernel launchers, which check every launch description the host produces."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2508_12407_amd", "csrc")


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs the host C++ compiler")
def test_host_runtime_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_check")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
           os.path.join(CSRC, "zz_api.cpp"), os.path.join(CSRC, "zz_transport.cpp"),
           os.path.join(ROOT, "tests", "host_runtime_sanitized.cpp"), "-o", exe]
    b = subprocess.run(cmd, capture_output=True, text=True)
    assert b.returncode == 0, b.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "failures: 0" in r.stdout


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs the host C++ compiler")
def test_host_time_of_a_decode_call_is_small(tmp_path, capsys):
    """The library's own host work per zz_decode_step call (optimised build, recorders instead of
    launches) stays far below a layer's GPU time (about 17 us per layer at 32k / batch 1)."""
    exe = str(tmp_path / "host_time")
    cmd = ["g++", "-std=c++17", "-O2", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
           "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, os.path.join(CSRC, "zz_api.cpp"),
           os.path.join(CSRC, "zz_transport.cpp"), os.path.join(ROOT, "tests", "host_runtime_sanitized.cpp"), "-o", exe]
    b = subprocess.run(cmd, capture_output=True, text=True)
    assert b.returncode == 0, b.stderr[-4000:]
    r = subprocess.run([exe, "--time"], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, (r.stdout, r.stderr)
    with capsys.disabled():
        print("\n" + r.stdout.strip())
    import re
    times = [float(x) for x in re.findall(r"layer (\d+) ns", r.stdout)]
    assert len(times) == 8
    assert max(times[:4]) < 2000        # equal lengths: well under 2 us per call
    assert max(times) < 20000           # 256 unequal lengths: the split plan's binary search
