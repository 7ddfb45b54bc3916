"""Are the pins of tests/test_oracle_pins.py sharp enough?  Each case below plants one plausible mistake in a
copy of oracle/kvc_oracle.c (a wrong divisor, the delta taken along the wrong axis, a swapped nibble, a
transposed index of the channel-pair order, ...), builds the copy and runs the pin tests against it in a
process of its own: the run has to fail.  The untouched copy has to pass the same way.  Everything happens on
the CPU and in a temporary folder; the oracle's own files are only read."""
import concurrent.futures
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "kvc_oracle.c")

# (name, text in the oracle, what it is replaced by)
MUTANTS = [
    ("scale divides by 128", "amax / 127.0f", "amax / 128.0f"),
    ("delta along tokens instead of channels", "int left = (i == 0) ? 0 : q[j * d + i - 1];",
     "int left = (j == 0) ? 0 : q[(j - 1) * d + i];"),
    ("zig-zag sends negative values to even codes", "v >= 0 ? 2 * v : -2 * v - 1", "v >= 0 ? 2 * v + 1 : -2 * v - 2"),
    ("zig-zag off by one on the negative side", "v >= 0 ? 2 * v : -2 * v - 1", "v >= 0 ? 2 * v : -2 * v + 1"),
    ("round half up instead of ties to even", "double r = nearbyint(p);", "double r = floor(p + 0.5);"),
    ("header nibbles swapped", "(g & 1) ? (code << 4) : code", "(g & 1) ? code : (code << 4)"),
    ("bits of a literal packet filled from the top of each byte", "(uint8_t)(bit << (p & 7))", "(uint8_t)(bit << (7 - (p & 7)))"),
    ("fallback only when strictly larger than INT8", "if (n >= int8_bytes)", "if (n > int8_bytes)"),
    ("inverse scale as 127 / amax instead of 1 / s", "*s_inv = 1.0f / *s;", "*s_inv = 127.0f / amax;"),
    ("un-zig-zag without the negation", "int delta = (int)(uu >> 1) ^ -(int)(uu & 1);", "int delta = (int)(uu >> 1) ^ (int)(uu & 1);"),
    ("dequantize with a scale that is slightly off", "float r = (float)q[i] * desc->scale;", "float r = (float)q[i] * desc->scale * 1.0001f;"),
    ("run packet under another code", "code = 9; /* run packet: one byte */", "code = 10;"),
    ("all-zero literal group at width 2", "if (w == 0) w = 1;", "if (w == 0) w = 2;"),
    ("page maximum taken over x instead of |x|", "float a = fabsf(kvo_half_to_float(x[i]));", "float a = kvo_half_to_float(x[i]);"),
    ("infinities not recognised, only NaN", "if ((x[i] & 0x7C00u) == 0x7C00u) return 1;", "if ((x[i] & 0x7FFFu) > 0x7C00u) return 1;"),
    ("header of an odd number of groups one byte short", "size_t hdr = (size_t)(G + 1) / 2;\n    memset(out, 0, hdr);", "size_t hdr = (size_t)G / 2;\n    memset(out, 0, hdr);"),
    ("payload padded to 8 bytes", "return (n + 15u) & ~(size_t)15u;", "return (n + 7u) & ~(size_t)7u;"),
    ("run packet also for groups of equal zeros under scheme 2", "if (with_runs && umax == 0) {", "if (umax == 0) {"),
    ("run test compares with the neighbour's first value", "if (ug[k] != ug[0]) all_equal = 0;", "if (ug[k] != u[0]) all_equal = 0;"),
    ("literal width from the first value instead of the maximum", "int w = bit_length(umax);", "int w = bit_length(ug[0] > 0 ? ug[0] : umax);"),
    ("scheme 2 written with run packets", "kvo_rle_pack(u, E, scheme != KVO_MODE_DELTA, tmp)", "kvo_rle_pack(u, E, 1, tmp)"),
    ("mode 4 keeps the delta step", "if (scheme == KVO_MODE_PACK)\n            kvo_zigzag_codes(q, E, u);", "if (0)\n            kvo_zigzag_codes(q, E, u);"),
    ("decoder sums deltas across token rows", "    for (int j = 0; j < N; ++j) {\n        int acc = 0;\n        for (int i = 0; i < d; ++i) {\n            unsigned uu = u[j * d + i];",
     "    int acc = 0;\n    for (int j = 0; j < N; ++j) {\n        for (int i = 0; i < d; ++i) {\n            unsigned uu = u[j * d + i];"),
    ("decoder saturates the running sum instead of wrapping it", "acc = (int8_t)(uint8_t)((acc + delta) & 0xFF);",
     "acc = acc + delta > 127 ? 127 : acc + delta < -128 ? -128 : acc + delta;"),
    ("decoder admits zero-run and run packets in a mode-2 page", "const int runs = mode != KVO_MODE_DELTA;", "const int runs = 1;"),
    ("decoder admits a packed page as large as its INT8 form", "if (nbytes >= kvo_pad16((size_t)E)) return KVO_ERR_CORRUPT;", "if (nbytes > kvo_pad16((size_t)E)) return KVO_ERR_CORRUPT;"),
    ("decoder accepts a payload with trailing bytes", "if (kvo_pad16(pos) != nbytes) goto corrupt;", "if (kvo_pad16(pos) > nbytes) goto corrupt;"),
    ("decoder accepts code 10 as a literal of width 8", "} else if (code >= 1 && code <= 8) {\n            int w = code;", "} else if (code >= 1) {\n            int w = code > 8 ? 8 : code;"),
    ("scale of an all-zero page is 1", "*s = 0.0f;\n        *s_inv = 0.0f;", "*s = 1.0f;\n        *s_inv = 0.0f;"),
    ("raw page reports the wrong size", "desc->n16 = (uint16_t)(E * 2 / 16);", "desc->n16 = (uint16_t)(E / 16);"),
    ("product rounded to binary32 before it is rounded to an integer", "double p = (double)kvo_half_to_float(x[i]) * (double)*s_inv;",
     "double p = (double)(float)((double)kvo_half_to_float(x[i]) * (double)*s_inv);"),
    ("mode 4 decoded as if it had a delta step", "if (mode == KVO_MODE_PACK) acc = 0;", ""),
    ("INT8 page of any size accepted", "if (nbytes != kvo_pad16((size_t)E)) return KVO_ERR_CORRUPT;", ""),
    ("raw page of any size accepted", "if (nbytes != (size_t)E * 2) goto bad;", ""),
    ("a refused page keeps what the output held", "bad:\n    memset(out, 0, (size_t)E * 2);", "bad:"),
    ("descriptor offsets of the second thread's pages not shifted", "desc[p].off += (uint64_t)total;", "desc[p].off += 0;"),
    ("a span that ends outside the pool is decoded", "ds->off + (uint64_t)ds->n16 * 16 > j->pool_bytes", "ds->off > j->pool_bytes"),
    ("a misaligned span is decoded", "if (ds->off % 16 != 0 || ", "if ("),
    ("gathered decode ignores the page ids", "&j->desc[j->page_ids ? j->page_ids[p] : p]", "&j->desc[p]"),
    ("mode 5 offered for 8-token pages", "static int chan_geometry_ok(int N, int d) {", "static int chan_geometry_ok(int N, int d) {\n    if (N == 8) return 1;"),
    ("FP16 subnormals scaled by 2^-25", "v = ldexp((double)m, -24);", "v = ldexp((double)m, -25);"),
    ("FP16 normals lose the hidden bit", "v = ldexp((double)(m + 1024), e - 25);", "v = ldexp((double)m, e - 25);"),
    ("FP16 exponent bias off by one", "v = ldexp((double)(m + 1024), e - 25);", "v = ldexp((double)(m + 1024), e - 24);"),
    ("rounding to FP16 truncates", "double m = nearbyint(ldexp(a, 10 - e)); /* in [1024, 2048] */", "double m = floor(ldexp(a, 10 - e));"),
    ("rounding to FP16 rounds ties away from zero", "double m = nearbyint(ldexp(a, 10 - e)); /* in [1024, 2048] */", "double m = floor(ldexp(a, 10 - e) + 0.5);"),
    ("a mantissa that rounds up to 2048 keeps its exponent", "        m = 1024.0;\n        e += 1;", "        m = 2047.0;"),
    ("values past 65504 stay finite", "if (e > 15) return (uint16_t)(sign | 0x7C00u);", "if (e > 15) return (uint16_t)(sign | 0x7BFFu);"),
    ("FP16 subnormal results rounded ties away", "double m = nearbyint(ldexp(a, 24));", "double m = floor(ldexp(a, 24) + 0.5);"),
    ("negative zero loses its sign on the way to FP16", "uint16_t sign = signbit(f) ? 0x8000u : 0u;", "uint16_t sign = f < 0 ? 0x8000u : 0u;"),
    ("mode 5 offered for d = 192", "(d / 8 <= 16 || (d / 8) % 16 == 0)", "(d / 8 <= 16 || (d / 8) % 8 == 0)"),
    ("thread ranges overlap by one page", "j->p1 = n_pages * (t + 1) / n_threads;", "j->p1 = n_pages * (t + 1) / n_threads + (t + 1 < n_threads ? 1 : 0);"),
    ("pool space check off by one page", "if ((uint64_t)total + j->used > pool_bytes) {", "if ((uint64_t)total > pool_bytes) {"),
    ("mode 5: groups in octet-major order", "return ((o / W) * 4 + j) * W + o % W;", "return o * 4 + j;"),
    ("mode 5: groups in pair-major order over the whole row", "return ((o / W) * 4 + j) * W + o % W;", "return (j * (d / 8)) + o;"),
    ("mode 5: runs of 8 octets instead of 16", "int W = d / 8 < 16 ? d / 8 : 16;", "int W = d / 8 < 8 ? d / 8 : 8;"),
    ("mode 5: token roles swapped inside a group", "int k = (t % 4) * 8 + (t / 4) * 2 + (c % 2);", "int k = (t / 4) * 8 + (t % 4) * 2 + (c % 2);"),
    ("mode 5: the decoder reads the pair's channels the other way round",
     "unsigned uu = u[32 * chan_group(c, d) + (t % 4) * 8 + (t / 4) * 2 + (c % 2)];",
     "unsigned uu = u[32 * chan_group(c, d) + (t % 4) * 8 + (t / 4) * 2 + 1 - (c % 2)];"),
]


def _run_pins(folder, text):
    os.makedirs(folder, exist_ok=True)
    src = os.path.join(folder, "kvc_oracle.c")
    with open(src, "w") as f:
        f.write(text)
    env = dict(os.environ, KVC_ORACLE_SRC=src, KVC_ORACLE_LIB=os.path.join(folder, "libkvc_oracle.so"))
    # the copy has to compile: a planted mistake that does not build would "fail" for the wrong reason
    subprocess.run([sys.executable, "-c", "from oracle import kvc_oracle; kvc_oracle.build(force=True)"], cwd=ROOT, env=env,
                   check=True, capture_output=True, timeout=300)
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                           "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not installed")
def test_every_planted_mistake_fails_a_pin(tmp_path):
    text = open(SRC).read()
    for name, old, new in MUTANTS:
        assert text.count(old) >= 1, f"'{name}': the line it changes is no longer in the oracle; update the case"
    control = _run_pins(str(tmp_path / "control"), text)
    assert control.returncode == 0, control.stdout[-2000:]
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
        runs = {name: ex.submit(_run_pins, str(tmp_path / f"m{i}"), text.replace(old, new, 1))
                for i, (name, old, new) in enumerate(MUTANTS)}
        survivors = []
        for name, fut in runs.items():
            r = fut.result()
            # a mistake is noticed by a failing pin (pytest exit status 1), by one of the oracle's own assertions (the
            # process aborts: -6) or, for a removed bounds check, by the crash it leads to (-11); any other status
            # means the run itself broke
            assert r.returncode in (0, 1, -6, -11), f"'{name}': the run broke instead of failing a pin\n{r.stdout[-1500:]}\n{r.stderr[-1500:]}"
            if r.returncode == 0:
                survivors.append(name)
    assert not survivors, f"no pin noticed: {survivors}"


# ------------------------------------------------------------------ the prefetch model (Algorithm 1)

MODEL = os.path.join(ROOT, "oracle", "prefetch_model.py")

MODEL_MUTANTS = [
    ("the half being filled is searched instead of the other one", "other = 1 - fill", "other = fill"),
    ("slots of the half being filled that are still to be overwritten count as resident", "for j2 in range(j):  # slots", "for j2 in range(k):  # slots"),
    ("the layer's offset into the pool is dropped", "phys = l * pool_blocks_per_layer + e", "phys = e"),
    ("the first block held in L1 is fetched all the same", "lb >= int(l1_first[s])", "lb > int(l1_first[s])"),
    ("a block already in its slot is transferred again", "if tags[fill, l, s, j] != phys:", "if True:"),
    ("window pieces one entry too long", "queue[i:i + omega]", "queue[i:i + omega + 1]"),
    ("a layer counts as ready one batch early", "return (done + omega - 1) // omega", "return done // omega"),
    ("slot reuse keeps duplicates", "keep.append(t in wanted and t not in seen)", "keep.append(t in wanted)"),
    ("window queue in sequence-major order", "    for l in range(layer_begin, layer_end):\n        for s in range(fetch.shape[1]):\n            for j in range(fetch.shape[2]):\n                if fetch[l, s, j] >= 0:",
     "    for s in range(fetch.shape[1]):\n        for l in range(layer_begin, layer_end):\n            for j in range(fetch.shape[2]):\n                if fetch[l, s, j] >= 0:"),
    ("window counts a layer's slots instead of its transfers", "                    per_layer[l] += 1", "                per_layer[l] += 1"),
    ("window queues slots that issued nothing", "if fetch[l, s, j] >= 0:\n                    queue.append", "if True:\n                    queue.append"),
    ("unbounded window reports every layer ready at once, also those behind an empty prefix", "return (done > 0).astype(np.int64)", "return np.ones_like(done, dtype=np.int64)"),
    ("a negative prediction is a bad index", "    if lb < 0:\n        return NO_BLOCK, False", "    if lb < 0:\n        return NO_BLOCK, True"),
    ("an empty table entry is a bad index", "    if e < 0:\n        return NO_BLOCK, False", "    if e < 0:\n        return NO_BLOCK, True"),
    ("positional policy: a prediction beyond the table is skipped silently", "                if lb >= max_blocks:\n                    bad_index = True", "                if lb >= max_blocks:\n                    bad_index = bad_index"),
    ("slot reuse takes the highest free slot", "j2 = keep.index(False)", "j2 = len(keep) - 1 - keep[::-1].index(False)"),
    ("an entry beyond the pool's blocks is taken as a block", "if e >= pbpl:\n        return NO_BLOCK, True", "if e > pbpl:\n        return NO_BLOCK, True"),
]

# runs the model's pin tests with the module text given on stdin standing in for oracle.prefetch_model
_RUNNER = """
import sys, types
sys.path.insert(0, {root!r})
import oracle
m = types.ModuleType("oracle.prefetch_model")
m.__file__ = "planted"
exec(compile(sys.stdin.read(), "planted_prefetch_model.py", "exec"), m.__dict__)
sys.modules["oracle.prefetch_model"] = m
oracle.prefetch_model = m
import pytest
sys.exit(int(pytest.main([{test!r}, "-x", "-q", "-p", "no:cacheprovider"])))
"""


def _run_model_pins(text):
    code = _RUNNER.format(root=ROOT, test=os.path.join(ROOT, "tests", "test_prefetch_model.py"))
    return subprocess.run([sys.executable, "-c", code], cwd=ROOT, input=text, capture_output=True, text=True, timeout=600)


def test_every_mistake_planted_in_the_prefetch_model_fails_a_pin():
    text = open(MODEL).read()
    for name, old, new in MODEL_MUTANTS:
        assert text.count(old) >= 1, f"'{name}': the line it changes is no longer in the model; update the case"
    control = _run_model_pins(text)
    assert control.returncode == 0, control.stdout[-2000:] + control.stderr[-2000:]
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
        runs = {name: ex.submit(_run_model_pins, text.replace(old, new)) for name, old, new in MODEL_MUTANTS}
        survivors = []
        for name, fut in runs.items():
            r = fut.result()
            assert r.returncode in (0, 1), f"'{name}': the run broke instead of failing a pin\n{r.stdout[-1500:]}\n{r.stderr[-1500:]}"
            if r.returncode == 0:
                survivors.append(name)
    assert not survivors, f"no pin noticed: {survivors}"
