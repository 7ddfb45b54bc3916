"""Structural rules of this build that a test can hold in place."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2512_11920_amd")


def _product_files():
    for base, _, files in os.walk(PKG):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp", ".c")):
                yield os.path.join(base, f)
    for base, _, files in os.walk(os.path.join(ROOT, "include")):
        for f in files:
            yield os.path.join(base, f)


def test_product_path_never_touches_the_oracle():
    """The oracle is test infrastructure: nothing in the package or the public header may import, include,
    link or name it, so no product call can be served by it."""
    for path in _product_files():
        text = open(path, errors="replace").read()
        assert not re.search(r"\boracle\b|kvc_oracle|kvo_|prefetch_model", text), path


def test_oracle_does_not_use_the_gpu_library():
    for base, _, files in os.walk(os.path.join(ROOT, "oracle")):
        for f in files:
            if f.endswith((".py", ".c", ".h")):
                text = open(os.path.join(base, f), errors="replace").read()
                assert "paper_2512_11920_amd" not in text and "libkvc.so" not in text and "hip" not in text.lower(), f


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "single-GPU" in r.stderr and not r.stdout.strip()


def test_no_cuda_compat_layers_in_kernels():
    for path in _product_files():
        if path.endswith((".hip", ".h")):
            text = open(path, errors="replace").read()
            assert "__HIP_PLATFORM" not in text and "cuda_runtime" not in text and "hipify" not in text.lower(), path


def test_traffic_lookup_refuses_a_summary_taken_on_other_sources(tmp_path, monkeypatch):
    """bench.py reports HBM traffic from a committed rocprofv3 summary only when the summary carries the
    fingerprint of the kernel sources in the tree."""
    sys.path.insert(0, ROOT)
    import bench

    fp = bench.kernel_fingerprint()
    assert re.fullmatch(r"[0-9a-f]{16}", fp) and fp == bench.kernel_fingerprint()
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    monkeypatch.setattr(bench, "kernel_fingerprint", lambda: fp)
    os.makedirs(tmp_path / "profiles")
    assert bench.read_traffic("w", "k_compress")[0] is None  # no summary at all
    (tmp_path / "profiles" / "hbm_traffic_w.txt").write_text(f"kernel_fingerprint: {fp}\nk_compress_traffic_bytes: 123\nk_decompress_traffic_bytes: 456\n")
    assert bench.read_traffic("w", "k_compress")[0] == 123 and bench.read_traffic("w", "k_decompress")[0] == 456
    (tmp_path / "profiles" / "hbm_traffic_w.txt").write_text("kernel_fingerprint: 0000000000000000\nk_compress_traffic_bytes: 123\n")
    val, src = bench.read_traffic("w", "k_compress")
    assert val is None and "other kernel sources" in src["note"]
