"""Randomized differential test: many pages from deliberately varied value distributions go through the
HIP library and the oracle; descriptors, payload bytes and decoded values must agree bit for bit."""
import os

import numpy as np
import pytest
import torch

from oracle import kvc_oracle as o
from paper_2512_11920_amd import kvc
from gpu_util import DEV, check_pool_invariants, compare_pages_with_oracle

pytestmark = pytest.mark.gpu


def _families(rng, n, N, d):
    """n pages, FP16 bit patterns, drawn from a mix of distributions."""
    out = np.zeros((n, N, d), np.float16)
    fam = rng.integers(0, 12, n)
    with np.errstate(over="ignore", invalid="ignore"):
        for i in range(n):
            f = fam[i]
            if f == 0:    # channel-scaled normal
                x = rng.standard_normal((N, d)) * np.exp(rng.uniform(0.05, 2.0) * rng.standard_normal(d))
            elif f == 1:  # heavy tails
                x = rng.standard_t(1.5, (N, d)) * rng.choice([0.01, 1, 30])
            elif f == 2:  # sparse
                x = rng.standard_normal((N, d)) * (rng.random((N, d)) < rng.choice([0.02, 0.1, 0.5]))
            elif f == 3:  # constant rows / ramps along channels (run packets)
                x = rng.integers(-3, 4, (N, 1)) * np.arange(d)[None, :] % 120 + rng.integers(-5, 6, (N, 1))
                x = x.astype(np.float64)
                x[rng.integers(0, N), rng.integers(0, d)] = 127 * rng.choice([-1, 1])
            elif f == 4:  # tiny magnitudes (FP16 subnormals)
                x = rng.standard_normal((N, d)) * 10.0 ** rng.uniform(-7.5, -4)
            elif f == 5:  # huge magnitudes
                x = rng.standard_normal((N, d)) * 10.0 ** rng.uniform(3, 4.3)
            elif f == 6:  # exact integer codes, amax = 127
                x = rng.integers(-127, 128, (N, d)).astype(np.float64)
                x[0, 0] = 127
            elif f == 7:  # small alphabets
                x = rng.choice([-1.0, 0.0, 1.0], (N, d), p=[0.1, 0.8, 0.1]) * rng.choice([1, 127, 0.003])
            elif f == 8:  # channel-correlated
                z = rng.standard_normal((N, d))
                rho = rng.choice([0.9, 0.99, 0.999])
                x = np.empty((N, d))
                x[:, 0] = z[:, 0]
                for j in range(1, d):
                    x[:, j] = rho * x[:, j - 1] + np.sqrt(1 - rho * rho) * z[:, j]
                x[:, rng.integers(0, d)] *= rng.choice([1, 10, 100])
            elif f == 9:  # token-constant channels with a few outliers
                x = np.repeat(rng.standard_normal((1, d)), N, axis=0) + 1e-3 * rng.standard_normal((N, d))
            elif f == 10:  # half the page zero (zero-run packets), the rest smooth
                x = np.cumsum(rng.integers(-2, 3, (N, d)), axis=1).astype(np.float64)
                x[rng.random(N) < 0.5] = 0
                x[0, 0] = 127
            else:          # raw bit patterns, NaN and Inf included
                out[i] = rng.integers(0, 65536, (N, d), dtype=np.uint16).view(np.float16)
                continue
            out[i] = np.clip(x, -65504, 65504).astype(np.float16)
    return out, fam


@pytest.mark.parametrize("N,d,n,scheme", [(16, 128, 40000, 3), (16, 128, 8000, 2), (16, 64, 8000, 3), (16, 256, 6000, 3),
                                          (16, 32, 3000, 3), (7, 128, 3000, 3), (32, 64, 3000, 2),
                                          (16, 128, 8000, 4), (16, 64, 3000, 4), (16, 256, 3000, 4), (5, 128, 2000, 4),
                                          # calls of at most 2048 pages take the encoder's low-latency launch shape
                                          (16, 128, 2048, 3), (16, 64, 2047, 3), (16, 256, 2048, 3), (16, 128, 1501, 4),
                                          (16, 64, 777, 2), (16, 256, 999, 1), (16, 128, 2049, 3),
                                          # mode 5: channel-pair groups (16 x 128 pages), both launch shapes
                                          (16, 128, 9000, 5), (16, 128, 2048, 5), (16, 128, 333, 5), (16, 256, 5000, 5), (16, 256, 1200, 5),
                                          (16, 64, 9000, 5), (16, 64, 2048, 5), (16, 64, 411, 5),
                                          # head dimensions that are not powers of two: token rows of 12, 20, 24, 28 lanes
                                          (16, 96, 3000, 3), (16, 160, 3000, 3), (16, 192, 3000, 3), (16, 224, 3000, 3),
                                          (16, 96, 2000, 4), (16, 192, 2000, 2), (8, 96, 2000, 3), (21, 192, 1500, 3), (3, 160, 2000, 3),
                                          # every other exact page shape, both launch shapes (large calls, calls of at most 2048 pages)
                                          (8, 64, 5000, 3), (8, 128, 4000, 2), (8, 192, 3000, 3), (8, 256, 3000, 4), (32, 32, 4000, 3),
                                          (32, 64, 3000, 3), (32, 96, 2500, 4), (32, 128, 2500, 3),
                                          (16, 32, 2000, 3), (16, 96, 1500, 3), (16, 160, 2048, 3), (16, 192, 1000, 3), (16, 224, 900, 4),
                                          (8, 64, 2000, 3), (8, 128, 1900, 4), (8, 192, 1000, 3), (8, 256, 800, 2), (32, 32, 2048, 4),
                                          (32, 64, 600, 3), (32, 96, 512, 3), (32, 128, 700, 2)])
def test_differential(N, d, n, scheme):
    # KVC_DIFF_SEED in the environment draws a different set of pages (for longer hunts)
    rng = np.random.default_rng(N * 1000 + d + scheme + 100003 * int(os.environ.get("KVC_DIFF_SEED", "0")))
    x, fam = _families(rng, n, N, d)
    print(f"[case] differential N={N} d={d} pages={n} scheme={scheme}", flush=True)
    xt = torch.from_numpy(x.reshape(-1, 1, N, d)).to(DEV)
    c = kvc.Codec(N, d, 1, scheme)
    c.alloc_pool(n, n * N * d * 2 + 64, DEV)
    c.compress_blocks(xt)
    out = torch.empty_like(xt)
    c.decompress_blocks(out)
    st = c.stats()
    assert st["rc"] == 0, st
    desc, pool = c.desc_numpy(), c.pool.cpu().numpy()
    check_pool_invariants(desc, st["pool_bytes_used"], pool.size)
    od, op = compare_pages_with_oracle(x.view(np.uint16), desc, pool, N, d, scheme)
    want, bad = o.decompress_pages(op, od, N, d, n_threads=8)
    assert bad == 0
    got = out.cpu().numpy().view(np.uint16).reshape(-1, N, d)
    if not np.array_equal(got, want):
        p = int(np.nonzero((got != want).any(axis=(1, 2)))[0][0])
        raise AssertionError(f"decoded page {p} (family {fam[p]}, mode {od['mode'][p]}) differs")
    modes = np.bincount(od["mode"], minlength=6)
    assert modes[0] > 0 and modes[1] > 0 and modes[scheme] > 0  # raw, fallback and packed pages all occurred


def _soak_pages(rng, n, N, d):
    """n pages drawn without Python loops: channel-scaled noise, channel-correlated walks (narrow widths,
    zero groups) and constant rows with offsets (run packets), mixed page by page."""
    kind = rng.integers(0, 3, n)
    noise = rng.standard_normal((n, N, d), dtype=np.float32) * np.exp(rng.standard_normal((n, 1, d), dtype=np.float32))
    walk = np.cumsum(rng.integers(-2, 3, (n, N, d), dtype=np.int8), axis=2, dtype=np.float32)
    walk[:, :, 0] += 100.0  # keeps the page maximum away from the walk's own range
    rows = np.broadcast_to(rng.integers(-60, 61, (n, N, 1)).astype(np.float32), (n, N, d)).copy()
    rows[:, 0, 0] = 127.0
    x = np.where((kind == 0)[:, None, None], noise, np.where((kind == 1)[:, None, None], walk, rows))
    return x.astype(np.float16)


_SOAK_CASES = [(16, d, sc) for d in (64, 128, 256) for sc in (2, 3, 4, "mixed")] + \
              [(N, d, sc) for (N, d) in ((8, 128), (32, 64), (16, 32), (4, 256)) for sc in (3, "mixed")] + [(16, 128, 5), (16, 256, 5), (16, 64, 5)] + \
              [(N, d, sc) for (N, d) in ((16, 96), (16, 160), (16, 192), (16, 224), (8, 96), (32, 96), (8, 192),
                                         (8, 64), (8, 256), (32, 32), (32, 128)) for sc in (3, "mixed")] + \
              [(N, d, sc) for (N, d) in ((7, 128), (24, 160), (3, 256), (15, 256), (21, 192), (100, 32), (4, 128), (12, 96),
                                         (18, 224), (40, 64)) for sc in (2, "mixed")]  # pages with a short last pass, one to eight passes


@pytest.mark.parametrize("N,d,scheme", _SOAK_CASES)
def test_every_kernel_instantiation_under_full_occupancy(N, d, scheme):
    """Instantiations of the kernels for exact page shapes (the compile-time scheme, the run-time scheme and
    the per-block scheme) and for pages with a short last pass, on enough pages that several workgroups share
    every compute unit, three launches each, every page compared with the oracle bit for bit."""
    n = 24576
    rng = np.random.default_rng(7000 + 31 * N + d + (9 if scheme == "mixed" else scheme) + 100003 * int(os.environ.get("KVC_DIFF_SEED", "0")))
    x = _soak_pages(rng, n, N, d)
    xt = torch.from_numpy(x.reshape(-1, 1, N, d)).to(DEV)
    if scheme == "mixed":
        n_modes = 6 if (N == 16 and d in (64, 128, 256)) else 5  # shapes that have mode 5 take it per block too
        per_block = rng.integers(0, n_modes, n).astype(np.uint8)
        bs = torch.from_numpy(per_block).to(DEV)
        od = np.zeros(n, o.DESC_DTYPE)
        chunks, off = [], 0
        for sc in range(n_modes):
            idx = np.nonzero(per_block == sc)[0]
            dd, pp = o.compress_pages(x[idx].view(np.uint16), N, d, sc, n_threads=16)
            dd = dd.copy()
            dd["off"] += off
            od[idx] = dd
            chunks.append(pp)
            off += pp.size
        op = np.concatenate(chunks)
    else:
        bs = None
        od, op = o.compress_pages(x.view(np.uint16), N, d, scheme, n_threads=16)
    want, bad = o.decompress_pages(op, od, N, d, n_threads=16)
    assert bad == 0
    c = kvc.Codec(N, d, 1, 3 if scheme == "mixed" else scheme)
    c.alloc_pool(n, n * N * d * 2 + 64, DEV)
    out = torch.empty_like(xt)
    for launch in range(3):
        c.reset_pool()
        c.compress_blocks(xt, block_scheme=bs)
        out.zero_()
        c.decompress_blocks(out)
        st = c.stats()
        assert st["rc"] == 0, st
        desc, pool = c.desc_numpy(), c.pool.cpu().numpy()
        assert np.array_equal(desc["mode"], od["mode"]) and np.array_equal(desc["n16"], od["n16"])
        assert np.array_equal(desc["scale"].view(np.uint32), od["scale"].view(np.uint32))
        size = od["n16"].astype(np.int64) * 16
        start = np.concatenate([[0], np.cumsum(size)[:-1]])
        got = pool[np.repeat(desc["off"].astype(np.int64) - start, size) + np.arange(size.sum())]
        ref = op[np.repeat(od["off"].astype(np.int64) - start, size) + np.arange(size.sum())]
        if not np.array_equal(got, ref):
            badp = np.unique(np.searchsorted(np.cumsum(size), np.nonzero(got != ref)[0], side="right"))
            raise AssertionError(f"launch {launch}: payload bytes differ in {badp.size} pages, first {badp[:8]}")
        assert np.array_equal(out.cpu().numpy().view(np.uint16).reshape(-1, N, d), want), f"launch {launch}: decoded values differ"


def _shape_pages(rng, n, N, d):
    x = _soak_pages(rng, n, N, d)
    x[0] = 0                                         # all zero
    x[1] = 0
    x[1, N - 1, d - 1] = -3.5                        # one element, the page's last
    x[2].view(np.uint16)[N // 2, d // 3] = 0x7E00    # a NaN: stored raw
    x[3] = np.float16(2.0)                           # every delta but the rows' first is zero
    x[4] = (np.arange(N * d).reshape(N, d) % 251).astype(np.float16)
    return x


@pytest.mark.parametrize("d", [32, 64, 96, 128, 160, 192, 224, 256])
def test_every_page_shape(d):
    """Every accepted token count for this channel count (N * d <= 4096): pages that fill their last pass of
    512 elements and pages that do not, with one to eight passes, an odd and an even number of packet
    groups.  Two requested modes per shape, both launch shapes of the encoder over the sweep."""
    for N in range(1, 4096 // d + 1):
        rng = np.random.default_rng(50000 + 97 * N + d)
        n = 2100 if N % 7 == 3 else 160  # some shapes with more than 2048 pages: the large-call launch shape
        x = _shape_pages(rng, n, N, d)
        xt = torch.from_numpy(x.reshape(-1, 1, N, d)).to(DEV)
        for scheme in (3, (N + d // 32) % 5):
            print(f"[case] page shape N={N} d={d} pages={n} scheme={scheme}", flush=True)
            c = kvc.Codec(N, d, 1, scheme)
            c.alloc_pool(n, n * N * d * 2 + 64, DEV)
            c.compress_blocks(xt)
            out = torch.full_like(xt, 7.0)
            c.decompress_blocks(out)
            st = c.stats()
            assert st["rc"] == 0, (N, d, scheme, st)
            desc, pool = c.desc_numpy(), c.pool.cpu().numpy()
            check_pool_invariants(desc, st["pool_bytes_used"], pool.size)
            od, op = compare_pages_with_oracle(x.view(np.uint16), desc, pool, N, d, scheme)
            want, bad = o.decompress_pages(op, od, N, d, n_threads=8)
            assert bad == 0
            assert np.array_equal(out.cpu().numpy().view(np.uint16).reshape(-1, N, d), want), (N, d, scheme)
