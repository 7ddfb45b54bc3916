"""Run by tests/test_gpu_debug_bounds.py in a process of its own: the parity cases through the
bounds-checking build of the library (libkvc_dbg.so, compiled with -DKVC_DEBUG_BOUNDS=1).  Every LDS index
and pool span the kernels compute is then checked on the device; a violation sets status bit 8."""
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))
from paper_2512_11920_amd import build, kvc  # noqa: E402

kvc.LIB_PATH = build.LIB_DEBUG
from oracle import kvc_oracle as o  # noqa: E402
import test_gpu_differential as td  # noqa: E402
import test_gpu_parity as tp  # noqa: E402

DEV = "cuda:0"
n_cases = 0
for N, d in ((16, 128), (16, 64), (16, 256), (16, 96), (16, 224), (8, 192), (32, 32), (8, 32), (5, 160)):
    rng = np.random.default_rng(900 + N + d)
    special = tp._special_pages(N, d, rng)
    families, _ = td._families(rng, 1500, N, d)
    x = np.concatenate([special, families])
    for scheme in ((3, 2, 4, 5) if (N == 16 and d in (64, 128, 256)) else (3, 2, 4)):
        print(f"[case] bounds-checking build N={N} d={d} scheme={scheme} pages={x.shape[0]}", flush=True)
        xt = torch.from_numpy(x.reshape(-1, 1, N, d)).to(DEV)
        c = kvc.Codec(N, d, 1, scheme)
        c.alloc_pool(x.shape[0], x.shape[0] * N * d * 2 + 64, DEV)
        c.compress_blocks(xt)
        out = torch.empty_like(xt)
        c.decompress_blocks(out)
        st = c.stats()
        assert st["status"] == 0, f"status {st['status']:#x}: bit 8 = an index or span left its bounds"
        od, op = o.compress_pages(x.view(np.uint16), N, d, scheme, n_threads=8)
        desc = c.desc_numpy()
        assert np.array_equal(desc["mode"], od["mode"]) and np.array_equal(desc["n16"], od["n16"])
        want, bad = o.decompress_pages(op, od, N, d, n_threads=8)
        assert bad == 0 and np.array_equal(out.cpu().numpy().view(np.uint16).reshape(-1, N, d), want)
        n_cases += 1
# one requested mode per block: the encoder instantiations that read the mode of every page (0..5 where the
# shape has mode 5, 0..4 elsewhere), decoded values against the oracle's for the same modes
for N, d in ((16, 64), (16, 128), (16, 256), (16, 96), (8, 64)):
    rng = np.random.default_rng(1300 + N + d)
    x = td._soak_pages(rng, 3000, N, d)
    n_modes = 6 if (N == 16 and d in (64, 128, 256)) else 5
    per_block = rng.integers(0, n_modes, x.shape[0]).astype(np.uint8)
    print(f"[case] bounds-checking build N={N} d={d} one of {n_modes} modes per block, pages={x.shape[0]}", flush=True)
    xt = torch.from_numpy(x.reshape(-1, 1, N, d)).to(DEV)
    c = kvc.Codec(N, d, 1, 3)
    c.alloc_pool(x.shape[0], x.shape[0] * N * d * 2 + 64, DEV)
    c.compress_blocks(xt, block_scheme=torch.from_numpy(per_block).to(DEV))
    out = torch.empty_like(xt)
    c.decompress_blocks(out)
    st = c.stats()
    assert st["status"] == 0, f"status {st['status']:#x}: bit 8 = an index or span left its bounds"
    desc = c.desc_numpy()
    got = out.cpu().numpy().view(np.uint16).reshape(-1, N, d)
    for sc in range(n_modes):
        idx = np.nonzero(per_block == sc)[0]
        od, op = o.compress_pages(x[idx].view(np.uint16), N, d, sc, n_threads=8)
        assert np.array_equal(desc["mode"][idx], od["mode"]) and np.array_equal(desc["n16"][idx], od["n16"])
        want, bad = o.decompress_pages(op, od, N, d, n_threads=8)
        assert bad == 0 and np.array_equal(got[idx], want)
    n_cases += 1
# pages with a short last pass: for every channel count the smallest, an odd, a middle and the largest token count
for d in (32, 64, 96, 128, 160, 192, 224, 256):
    n_max = 4096 // d
    for N in sorted({1, 3, n_max // 2 + 1, n_max - 1, n_max}):
        rng = np.random.default_rng(7 * N + d)
        x = td._shape_pages(rng, 300, N, d)
        for scheme in (3, (N + d // 32) % 5):
            print(f"[case] bounds-checking build N={N} d={d} scheme={scheme} pages={x.shape[0]}", flush=True)
            xt = torch.from_numpy(x.reshape(-1, 1, N, d)).to(DEV)
            c = kvc.Codec(N, d, 1, scheme)
            c.alloc_pool(x.shape[0], x.shape[0] * N * d * 2 + 64, DEV)
            c.compress_blocks(xt)
            out = torch.empty_like(xt)
            c.decompress_blocks(out)
            st = c.stats()
            assert st["status"] == 0, f"status {st['status']:#x}: bit 8 = an index or span left its bounds"
            od, op = o.compress_pages(x.view(np.uint16), N, d, scheme, n_threads=8)
            want, bad = o.decompress_pages(op, od, N, d, n_threads=8)
            assert bad == 0 and np.array_equal(out.cpu().numpy().view(np.uint16).reshape(-1, N, d), want)
            n_cases += 1
# the prefetch window's queue builder and engines (these tests end with status == 0, which includes bit 8)
import test_gpu_prefetch as tpf  # noqa: E402

for omega, geom in ((5, (16, 128, 4, 5, 8, 4, 48, 200)), (16, (8, 32, 2, 5, 8, 4, 48, 200)), (4096, (16, 32, 1, 48, 16, 5, 400, 800))):
    tpf.test_window_prefetch_matches_unbounded_and_model(omega, geom)
    n_cases += 1
print(f"debug-bounds ok: {n_cases} cases", flush=True)
