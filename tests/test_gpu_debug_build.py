"""The bounds-checking debug build of the library (libzz_debug.so: same sources, -DZZ_DEBUG_BOUNDS) run
over every kind of cache-slot write, in a child process that loads it instead of the regular build."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_debug_build_refuses_no_slot_write_and_builds_the_same_caches():
    lib = os.path.join(ROOT, "paper_2508_12407_amd", "libzz_debug.so")
    assert os.path.exists(lib), "build with __graft_entry__.build()"
    env = dict(os.environ, ZZ_LIBRARY="libzz_debug.so", PYTHONPATH=ROOT)
    r = subprocess.run([sys.executable, "-u", os.path.join(ROOT, "tests", "debug_build_check.py")], env=env,
                       capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-3000:])
    assert "refused slot writes: 0" in r.stdout
