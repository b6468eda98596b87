"""The C ABI used from a plain C++ program (tests/c_abi_client.cpp): hipMalloc memory, a HIP
stream, no Python and no torch in the process.  The program checks its own results against
closed forms (uniform keys give the mean of the attended positions) and prints PASS."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLIENT = os.path.join(ROOT, "paper_2508_12407_amd", "zz_c_abi_client")


def test_client_is_built_and_links_against_the_library():
    assert os.path.exists(CLIENT), "run `python __graft_entry__.py` first"
    out = subprocess.run(["ldd", CLIENT], capture_output=True, text=True).stdout
    assert "libzz.so" in out and "not found" not in out.split("libzz.so")[1].splitlines()[0], out


@pytest.mark.gpu
def test_c_client_runs_prefill_decode_and_fused_step_on_the_gpu():
    r = subprocess.run([CLIENT], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.strip().endswith("PASS"), (r.returncode, r.stdout[-2000:], r.stderr[-2000:])
