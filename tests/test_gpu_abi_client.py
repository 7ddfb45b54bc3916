"""The C ABI used from a plain C++ program: no Python binding, no torch, only the HIP runtime and
include/kvc.h.  The program (tests/abi_client.cpp, built by __graft_entry__.build()) runs compress,
stats, decompress and gather-decompress and checks the quantizer's error bound itself."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

_BIN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "abi_client")


def test_c_abi_from_a_program_without_python_or_torch():
    if not os.path.exists(_BIN):  # normally built by __graft_entry__.build(); a few seconds with hipcc
        from paper_2512_11920_amd import build

        build.build_client()
    assert os.path.exists(_BIN), "tests/abi_client is not built; run `python __graft_entry__.py`"
    r = subprocess.run([_BIN], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0, (r.returncode, r.stdout[-2000:], r.stderr[-2000:])
    assert "abi client ok" in r.stdout
    assert "error bound holds on all 4096 pages" in r.stdout
