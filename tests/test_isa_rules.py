"""Rules for the generated gfx950 code that a GPU run cannot be trusted to catch.

(1) 64-bit shifts by a per-lane amount.  One build of one encoder instantiation wrote wrong payload bytes
for a few pages in a thousand, only when workgroups shared a compute unit, and every recompile that moved
registers made it vanish; the working hypothesis (not established from evidence kept in this tree) is that
v_lshlrev_b64 / v_lshrrev_b64 misread a shift count held in the last VGPR of the wave's allocation.  Which
register holds the count is the compiler's choice, so the kernels contain no 64-bit shift by a register
amount at all (v_ashrrev_i64 is kept out with them): counts that are immediates or scalar registers are fine.

(2) Workgroup barriers of the prefetch window's engines stay out of nested loops (see the test)."""
import concurrent.futures
import os
import re

import pytest

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.fixture(scope="module")
def asm(tmp_path_factory):
    """gfx950 assembly of every compilation unit that holds kernels, by unit name."""
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not installed")
    from paper_2512_11920_amd import build

    d = tmp_path_factory.mktemp("asm")
    units = [(src, defs, obj) for src, defs, obj in build.UNITS if src != "kvc_api.hip"]
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        futs = {obj: ex.submit(build.compile_unit, src, defs, str(d / (obj + ".s")), (), True) for src, defs, obj in units}
        texts = {obj: open(f.result()).read() for obj, f in futs.items()}
    for name, text in texts.items():
        assert ".amdgcn_target" in text and "gfx950" in text, name
    return texts


def test_no_64_bit_shift_by_a_vector_register(asm):
    for name, text in asm.items():
        hits = re.findall(r"^\s*v_(?:lshlrev_b64|lshrrev_b64|ashrrev_i64)\s+v\[\d+:\d+\],\s*v\d+,.*$", text, flags=re.M)
        assert not hits, f"{name}: {len(hits)} 64-bit shifts by a VGPR amount, e.g. {hits[0].strip()}"


def test_no_kernel_spills_registers_to_memory(asm):
    """Every kernel keeps its working set in registers: scratch (private memory) use would mean spills,
    which cost HBM traffic the byte accounting does not know about."""
    n = 0
    for name, text in asm.items():
        for m in re.finditer(r"\.name:\s+(\S+).*?\.private_segment_fixed_size:\s*(\d+)", text, flags=re.S):
            n += 1
            if "k_prefetch_plan" in m.group(1):
                continue  # the planner keeps up to 32 predictions and both halves' tags per thread; it moves no pages
            assert int(m.group(2)) == 0, f"{name}: {m.group(1)} uses {m.group(2)} bytes of scratch memory"
    assert n > 20


def test_window_engines_keep_their_barriers_out_of_nested_loops(asm):
    """The transfer engines of the prefetch window loop over queue entries with workgroup barriers in the
    loop body and single-lane bookkeeping between them.  The compiler must lay that out as one loop whose
    barriers every wave meets with all lanes: a barrier inside a loop nested in the engines' loop means
    the single-lane work was hoisted across the back edge and the other lanes run ahead to the next
    barrier (the workgroup then waits for ever).  Checked on the generated code: in every window kernel
    all s_barrier instructions sit at loop depth 0 or 1."""
    seen = 0
    for name, text in asm.items():
        lines = text.split("\n")
        for st in [i for i, l in enumerate(lines) if re.match(r"^_Z\w*k_decompress_window\w*:", l)]:
            seen += 1
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
                    assert depth <= 1, f"{name}: {lines[st][:60]}: s_barrier at loop depth {depth} (line {i - st})"
                i += 1
            assert n_barriers >= 4, "the engine loop should hold two barriers per turn plus two in the prologue"
    assert seen >= 64 + 16, "window kernels of every page shape: 64 with a run-time token count, 16 exact"
