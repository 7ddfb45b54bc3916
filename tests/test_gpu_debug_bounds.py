"""The bounds-checking build of the kernels (-DKVC_DEBUG_BOUNDS=1: every LDS slot index and pool span
is checked on the device, a violation sets status bit 8 instead of being executed silently) runs the
special pages and the randomized families of every kind of geometry, in a process of its own so that
this process keeps the ordinary library."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.timeout(600)
def test_parity_cases_stay_inside_their_bounds():
    from paper_2512_11920_amd import build

    if not os.path.exists(build.LIB_DEBUG):  # normally built by __graft_entry__.build()
        build.build_debug()
    p = subprocess.run([sys.executable, "-u", os.path.join(HERE, "debug_bounds_run.py")], capture_output=True, text=True, timeout=550)
    print(p.stdout[-3000:], flush=True)
    assert p.returncode == 0, p.stderr[-3000:]
    assert "debug-bounds ok" in p.stdout
