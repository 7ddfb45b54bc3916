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


@pytest.mark.parametrize("source", ["kvc_page16.hip", "kvc_kernels.hip"])
def test_window_engines_keep_their_barriers_out_of_nested_loops(source, tmp_path):
    """The transfer engines of the prefetch window loop over queue entries with workgroup barriers in the
    loop body and single-lane bookkeeping between them.  The compiler must lay that out as one loop whose
    barriers every wave meets with all lanes: a barrier inside a loop nested in the engines' loop means
    the single-lane work was hoisted across the back edge and the other lanes run ahead to the next
    barrier (the workgroup then waits for ever).  Checked on the generated code: in every window kernel
    all s_barrier instructions sit at loop depth 0 or 1."""
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not installed")
    out = tmp_path / (source + ".s")
    from paper_2512_11920_amd.build import HIPCC_FLAGS

    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    subprocess.run([HIPCC, *flags, "-S", "--cuda-device-only", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                    "-o", str(out), os.path.join(CSRC, source)], check=True, capture_output=True)
    lines = out.read_text().split("\n")
    kernels = [i for i, l in enumerate(lines) if re.match(r"^_Z\w*k_decompress_window\w*:", l)]
    assert kernels, "no window kernel found in the generated code"
    for st in kernels:
        en = next(i for i in range(st, len(lines)) if "s_endpgm" in lines[i])
        depth, n_barriers = 0, 0
        i = st + 1
        while i <= en:
            l = lines[i]
            if re.match(r"^\.LBB\d+_\d+:", l) or re.match(r"^; %bb\.\d+:", l):
                # depth of this block: the largest Depth= named in its label comment lines
                ds = [int(x) for x in re.findall(r"Depth=(\d+)", l)]
                j = i + 1
                while j <= en and lines[j].lstrip().startswith(";") and not re.match(r"^; %bb\.", lines[j]):
                    if "This" in lines[j] and "Loop Header" in lines[j]:
                        ds += [int(x) for x in re.findall(r"Depth=(\d+)", lines[j])]
                    j += 1
                depth = max(ds) if ds else 0
            elif "s_barrier" in l:
                n_barriers += 1
                assert depth <= 1, f"{lines[st][:60]}: s_barrier at loop depth {depth} (line {i - st})"
            i += 1
        assert n_barriers >= 4, "the engine loop should hold two barriers per turn plus two in the prologue"
