"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer: a second build of oracle/kvc_oracle.c,
linked into a small driver program (tests/oracle_san_driver.c), runs the hand-worked pages, the brute-force
single-group pages, pages of every mode and geometry the tests use, and corrupted descriptors and payloads.
The run must end without a sanitizer report and must return exactly what the ordinary build returns."""
import itertools
import json
import os
import struct
import subprocess

import numpy as np
import pytest

from oracle import kvc_oracle as o

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "oracle_san_driver")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-pthread", "-Wall", "-Wextra", "-o", exe,
           os.path.join(ROOT, "oracle", "kvc_oracle.c"), os.path.join(HERE, "oracle_san_driver.c"), "-lm"]
    subprocess.run(cmd, check=True)
    return exe


def _run(driver, records, tmp_path):
    """records: list of dicts (kind 1: x, N, d, scheme, threads; kind 2: desc, pool, N, d, threads).
    -> list of results read back from the sanitized run."""
    fin, fout = tmp_path / "cases.bin", tmp_path / "results.bin"
    with open(fin, "wb") as f:
        for r in records:
            if r["kind"] == 1:
                x = np.ascontiguousarray(r["x"]).view(np.uint16).reshape(-1, r["N"], r["d"])
                f.write(struct.pack("<6iq", 1, r["N"], r["d"], r["scheme"], x.shape[0], r.get("threads", 1), 0))
                f.write(x.tobytes())
            else:
                desc, pool = np.ascontiguousarray(r["desc"], o.DESC_DTYPE), np.ascontiguousarray(r["pool"], np.uint8)
                f.write(struct.pack("<6iq", 2, r["N"], r["d"], 0, desc.size, r.get("threads", 1), pool.size))
                f.write(desc.tobytes())
                f.write(pool.tobytes())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    p = subprocess.run([driver, str(fin), str(fout)], capture_output=True, text=True, env=env, timeout=600)
    assert p.returncode == 0 and "Sanitizer" not in p.stderr and "runtime error" not in p.stderr, p.stderr[-4000:]
    assert f"{len(records)} records" in p.stdout
    buf = open(fout, "rb").read()
    pos, results = 0, []
    for r in records:
        used, bad = struct.unpack_from("<qq", buf, pos)
        pos += 16
        res = {"used": used, "bad": bad}
        if r["kind"] == 1:
            n = np.asarray(r["x"]).size // (r["N"] * r["d"])
            res["desc"] = np.frombuffer(buf, o.DESC_DTYPE, n, pos)
            pos += 16 * n
            res["pool"] = np.frombuffer(buf, np.uint8, used, pos)
            pos += used
        else:
            n = np.asarray(r["desc"]).size
        res["out"] = np.frombuffer(buf, np.uint16, n * r["N"] * r["d"], pos).reshape(n, r["N"], r["d"])
        pos += 2 * n * r["N"] * r["d"]
        results.append(res)
    assert pos == len(buf)
    return results


def _check_against_plain_build(records, results):
    for r, res in zip(records, results):
        if r["kind"] == 1:
            od, op = o.compress_pages(r["x"], r["N"], r["d"], r["scheme"])
            assert np.array_equal(od, res["desc"]) and np.array_equal(op, res["pool"])
            want, bad = o.decompress_pages(op, od, r["N"], r["d"])
        else:
            want, bad = o.decompress_pages(r["pool"], r["desc"], r["N"], r["d"])
        assert bad == res["bad"] and np.array_equal(want, res["out"])


def test_handworked_bruteforce_and_mixed_pages_run_clean(driver, tmp_path):
    rng = np.random.default_rng(5)
    records = []
    for cs in json.load(open(os.path.join(HERE, "golden", "kvc1_handworked.json")))["cases"]:
        x = np.frombuffer(bytes.fromhex(cs["x_fp16_le_hex"]), np.uint16)
        records.append(dict(kind=1, x=x, N=cs["N"], d=cs["d"], scheme=cs["scheme"]))
    # every single-group page whose first 8 codes come from {-1, 0, 1} (the rest zero), amax pinned by a 127
    vals = np.array(list(itertools.product((-1.0, 0.0, 1.0), repeat=8)), np.float16)
    x = np.zeros((vals.shape[0], 1, 64), np.float16)
    x[:, 0, :8] = vals
    x[:, 0, 40] = 127
    for scheme in (3, 2, 4):
        records.append(dict(kind=1, x=x, N=1, d=64, scheme=scheme, threads=3))
    # pages of every mode and of the geometries the GPU tests use, NaN/Inf pages included
    for N, d in ((16, 128), (16, 64), (16, 256), (16, 96), (16, 224), (8, 32), (5, 160), (1, 32), (32, 128)):
        p = (rng.standard_normal((40, N, d)) * np.exp(rng.standard_normal((40, 1, d)))).astype(np.float16)
        p[3] = 0
        p[4, 0, 0] = np.inf
        p[5, N - 1, d - 1] = np.nan
        p[6] = np.cumsum(rng.integers(-2, 3, (N, d)), axis=1).clip(-100, 100)
        p[7, :, :] = 3.0
        for scheme in ((0, 1, 2, 3, 4, 5) if N == 16 and d != 224 else (0, 1, 2, 3, 4)):  # mode 5: 16-token pages, whole runs of octets
            records.append(dict(kind=1, x=p, N=N, d=d, scheme=scheme, threads=2))
    results = _run(driver, records, tmp_path)
    _check_against_plain_build(records, results)
    for cs, res in zip(json.load(open(os.path.join(HERE, "golden", "kvc1_handworked.json")))["cases"], results):
        assert res["pool"].tobytes().hex() == cs["payload_hex"] and int(res["desc"]["mode"][0]) == cs["mode"]


def test_corrupt_inputs_are_rejected_without_touching_memory_out_of_bounds(driver, tmp_path):
    rng = np.random.default_rng(6)
    records = []
    for N, d, scheme in ((16, 128, 3), (16, 128, 5), (16, 64, 2), (8, 96, 4), (16, 256, 3)):
        x = (rng.standard_normal((24, N, d)) * np.exp(rng.standard_normal((24, 1, d)))).astype(np.float16)
        x[:, :, 3] *= 30
        od, op = o.compress_pages(x, N, d, scheme)
        # descriptor faults: unknown and invalid modes, sizes one unit off, spans beyond the pool, odd offsets
        for field, fn in (("mode", lambda v: 0xFF), ("mode", lambda v: 7), ("mode", lambda v: (int(v) + 1) % 6),
                          ("n16", lambda v: int(v) - 1), ("n16", lambda v: int(v) + 1), ("n16", lambda v: 0), ("n16", lambda v: 0xFFFF),
                          ("off", lambda v: int(v) + 8), ("off", lambda v: op.size), ("off", lambda v: 2 ** 63), ("scale", lambda v: np.nan)):
            d2 = od.copy()
            for i in range(0, d2.size, 3):
                d2[field][i] = fn(d2[field][i])
            records.append(dict(kind=2, desc=d2, pool=op, N=N, d=d, threads=2))
        # payload faults: random bytes, header nibbles above 9, a truncated pool
        for trial in range(6):
            p2 = op.copy()
            idx = rng.integers(0, p2.size, 200)
            p2[idx] = rng.integers(0, 256, idx.size)
            records.append(dict(kind=2, desc=od, pool=p2, N=N, d=d))
        p2 = op.copy()
        p2[od["off"].astype(np.int64)] = 0xAA
        records.append(dict(kind=2, desc=od, pool=p2, N=N, d=d))
        records.append(dict(kind=2, desc=od, pool=op[: op.size // 2], N=N, d=d))
        records.append(dict(kind=2, desc=od, pool=rng.integers(0, 256, op.size).astype(np.uint8), N=N, d=d))
    results = _run(driver, records, tmp_path)
    _check_against_plain_build(records, results)
    assert sum(r["bad"] for r in results) > 100  # the faults were faults
