"""Input generator pins and the oracle's compression ratio on the synthetic distributions.
The paper's 3.21x / [2.5, 4.0] (Table 9, Section 3.5.2) was measured on real LLaMA-2 KV caches
and is parity-unpinned here; these tests fix what can be fixed and print the rest."""
import hashlib
import os

import numpy as np

from oracle import kvc_oracle as o
from paper_2512_11920_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_tiny_input_bytes_are_reproducible():
    want = [l.strip() for l in open(os.path.join(GOLD, "tiny_input_sha256.txt")) if l.strip() and l[0] != "#"][0]
    x = synth.cache_numpy(synth.CONFIGS["tiny"])
    assert x.shape == (1, 2, 16, 4, 16, 64) and x.dtype == np.float16
    assert hashlib.sha256(x.tobytes()).hexdigest() == want


def test_config_geometry_matches_the_workload_table():
    c = synth.CONFIGS
    assert c["tiny"].n_pages == 128 and c["tiny"].nbytes == 262144
    assert c["7b_layer"].n_pages == 65536
    assert c["7b_full"].n_pages == 8388608 and round(c["7b_full"].nbytes / 1e9, 2) == 34.36
    assert c["70b_gqa"].n_pages == 5242880 and round(c["70b_gqa"].nbytes / 1e9, 2) == 21.47


def test_distribution_has_key_outlier_channels_only():
    sh = synth.KVShape("probe", 4, 8, 128, 64, 1)
    cs = np.stack([synth.channel_scales(sh, l) for l in range(4)])
    logk = np.log(cs[:, 0]).ravel()
    logv = np.log(cs[:, 1]).ravel()
    assert abs(logv.mean()) < 0.05 and abs(logv.std() - 0.5) < 0.05
    frac = (logk > 1.7).mean()  # x10 outliers sit near ln(10) = 2.3 above the bulk
    assert 0.005 < frac < 0.04
    x = synth.layer_numpy(sh, 0).astype(np.float32)
    assert np.allclose(x[1].std(axis=(0, 2)), cs[0, 1], rtol=0.35)


def test_gather_pattern_is_a_permutation_and_predictions_in_range():
    pat = synth.gather_pattern(n_seq=16, k=8, seed=0)
    assert pat.lengths.min() >= 512 and pat.lengths.max() <= 8192
    used = pat.block_table[pat.block_table >= 0]
    assert used.size == pat.pool_blocks_per_layer == int(pat.n_blocks.sum())
    assert np.array_equal(np.sort(used), np.arange(used.size))
    for step in (0, 1, 999):
        pr = pat.predictions(step)
        assert pr.shape == (16, 8) and (pr >= 0).all() and (pr < pat.n_blocks[:, None]).all()
    assert not np.array_equal(pat.predictions(0), pat.predictions(1))
    assert np.array_equal(pat.predictions(5), pat.predictions(5))


def test_ratio_on_synthetic_llama_shaped_pages(capsys):
    sh = synth.KVShape("probe", 1, 8, 128, 1024, 1)
    x = synth.cache_numpy(sh)[0]
    rk = o.ratio(o.compress_pages(x[0], 16, 128, 3)[0], 2048)
    rv = o.ratio(o.compress_pages(x[1], 16, 128, 3)[0], 2048)
    desc, _ = o.compress_pages(x, 16, 128, 3)
    r = o.ratio(desc, 2048)
    with capsys.disabled():
        print(f"\n[ratio] synthetic i.i.d.-channel KV: K {rk:.3f}x  V {rv:.3f}x  K+V {r:.3f}x "
              f"(paper, real KV caches: 3.21x, band [2.5, 4.0])")
    # every finite page is at worst plain INT8: 4096 / (2048 + 16)
    assert (desc["mode"] != 0).all()
    assert min(rk, rv) >= 4096 / 2064 - 1e-9
    assert rk > rv  # outlier channels shrink the other keys' codes
    assert 2.0 < r < 2.6


def test_ratio_reaches_paper_band_on_channel_correlated_pages(capsys):
    """Delta coding exploits correlation along the channel index (Section 3.1, item v); the
    i.i.d. synthetic workload has none.  AR(1) along d with one x10 channel does."""
    rng = np.random.default_rng(0)
    rho = 0.95
    z = rng.standard_normal((64, 16, 128))
    y = np.zeros_like(z)
    y[..., 0] = z[..., 0]
    for i in range(1, 128):
        y[..., i] = rho * y[..., i - 1] + np.sqrt(1 - rho * rho) * z[..., i]
    y[..., 77] *= 10
    r3 = o.ratio(o.compress_pages(y.astype(np.float16), 16, 128, 3)[0], 2048)
    r2 = o.ratio(o.compress_pages(y.astype(np.float16), 16, 128, 2)[0], 2048)
    r1 = o.ratio(o.compress_pages(y.astype(np.float16), 16, 128, 1)[0], 2048)
    with capsys.disabled():
        print(f"\n[ratio] AR(1) rho=0.95 + outlier channel: INT8 {r1:.2f}x  +Delta {r2:.2f}x  +RLE {r3:.2f}x "
              f"(paper Table 9: 2.00 / 2.73 / 3.21)")
    assert 2.5 <= r3 <= 4.0 and r3 >= r2 > r1
