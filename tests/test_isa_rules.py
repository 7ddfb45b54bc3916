"""Rules for the generated gfx950 code that a GPU run cannot be trusted to catch.

On MI355X the 64-bit shift instructions v_lshlrev_b64 and v_lshrrev_b64 misread a shift count held in
the last VGPR of the wave's allocation when another wave shares the SIMD (found with one build of the
encoder and reproduced in a stand-alone kernel); v_ashrrev_i64 was not measured and is kept out with them.  Which register holds the count is the
compiler's choice, so the kernels must contain no 64-bit shift by a register amount at all: counts that
are immediates or scalar registers are fine."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2512_11920_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.parametrize("source", ["kvc_page16.hip", "kvc_kernels.hip"])
def test_no_64_bit_shift_by_a_vector_register(source, tmp_path):
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not installed")
    out = tmp_path / (source + ".s")
    from paper_2512_11920_amd.build import HIPCC_FLAGS

    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    subprocess.run([HIPCC, *flags, "-S", "--cuda-device-only", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                    "-o", str(out), os.path.join(CSRC, source)], check=True, capture_output=True)
    text = out.read_text()
    assert ".amdgcn_target" in text and "gfx950" in text
    hits = re.findall(r"^\s*v_(?:lshlrev_b64|lshrrev_b64|ashrrev_i64)\s+v\[\d+:\d+\],\s*v\d+,.*$", text, flags=re.M)
    assert not hits, f"{len(hits)} 64-bit shifts by a VGPR amount, e.g. {hits[0].strip()}"
