"""Randomized differential test: many pages from deliberately varied value distributions go through the
HIP library and the oracle; descriptors, payload bytes and decoded values must agree bit for bit."""
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
                                          (16, 128, 8000, 4), (16, 64, 3000, 4), (16, 256, 3000, 4), (5, 128, 2000, 4)])
def test_differential(N, d, n, scheme):
    rng = np.random.default_rng(N * 1000 + d + scheme)
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
    modes = np.bincount(od["mode"], minlength=5)
    assert modes[0] > 0 and modes[1] > 0 and modes[scheme] > 0  # raw, fallback and packed pages all occurred
