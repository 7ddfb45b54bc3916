"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element on
the same seeded inputs.  Bar: descriptors, codes, packed bitstreams, padding bit-exact; binary32
scales bit-exact; decoded FP16 bit-exact (the stated bar is <= 1 FP16 ulp; the arithmetic is the
same single-rounded product on both sides, so 0 is what is asserted)."""
import json
import os

import numpy as np
import pytest
import torch

from oracle import kvc_oracle as o
from paper_2512_11920_amd import kvc, synth
from gpu_util import (DEV, check_pool_invariants, compare_pages_with_oracle, gpu_compress, make_codec,
                      upload_oracle_pool)

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _say(msg):
    print(msg, flush=True)


def _roundtrip_case(x, N, d, ppb, scheme, name):
    _say(f"[case] {name}: pages={x.size // (N * d)} N={N} d={d} ppb={ppb} scheme={scheme}")
    xu = np.ascontiguousarray(x).view(np.uint16).reshape(-1, N, d)
    c, xt = gpu_compress(xu, N, d, ppb, scheme)
    st = c.stats()
    assert st["rc"] == 0 and st["status"] == 0, st
    desc = c.desc_numpy()
    pool = c.pool.cpu().numpy()
    check_pool_invariants(desc, st["pool_bytes_used"], pool.size)
    od, op = compare_pages_with_oracle(xu, desc, pool, N, d, scheme)
    assert st["pages"] == np.bincount(od["mode"], minlength=6).tolist() and st["pages_invalid"] == 0
    assert st["payload_bytes"] == op.size
    assert c.ratio() == pytest.approx(o.ratio(od, N * d))
    # decode GPU-made pool on the GPU
    out = torch.full_like(xt, float("nan"))
    c.decompress_blocks(out)
    torch.cuda.synchronize()
    want, bad = o.decompress_pages(op, od, N, d, n_threads=8)
    assert bad == 0
    got = out.cpu().numpy().view(np.uint16).reshape(-1, N, d)
    assert np.array_equal(got, want), f"decoded pages differ: {np.nonzero((got != want).any(axis=(1, 2)))[0][:10]}"
    assert c.stats()["status"] == 0
    # decode the ORACLE-made pool on the GPU (independent of the GPU encoder)
    c2 = kvc.Codec(N, d, ppb, scheme)
    upload_oracle_pool(c2, od, op)
    out2 = torch.full_like(xt, float("nan"))
    c2.decompress_blocks(out2)
    torch.cuda.synchronize()
    assert np.array_equal(out2.cpu().numpy().view(np.uint16).reshape(-1, N, d), want)
    assert c2.stats()["status"] == 0
    return od


@pytest.mark.parametrize("scheme", [3, 2, 1, 0, 4])
def test_tiny_config_all_pages(scheme):
    sh = synth.CONFIGS["tiny"]
    x = synth.cache_numpy(sh)  # [1][2][16][4][16][64]
    od = _roundtrip_case(x, 16, 64, 4, scheme, f"tiny/scheme{scheme}")
    if scheme == 3:
        assert set(np.unique(od["mode"])) <= {1, 3}


def test_handworked_pages_on_gpu():
    cases = json.load(open(os.path.join(GOLD, "kvc1_handworked.json")))["cases"]
    for cs in cases:
        x = np.frombuffer(bytes.fromhex(cs["x_fp16_le_hex"]), np.uint16)
        _say(f"[case] golden/{cs['name']}")
        c, xt = gpu_compress(x, cs["N"], cs["d"], 1, cs["scheme"])
        desc = c.desc_numpy()
        pool = c.pool.cpu().numpy()
        assert int(desc["mode"][0]) == cs["mode"] and int(desc["n16"][0]) == cs["n16"]
        assert f"{int(desc['scale'].view(np.uint32)[0]):08x}" == cs["scale_bits"]
        o0 = int(desc["off"][0])
        assert pool[o0:o0 + 16 * cs["n16"]].tobytes().hex() == cs["payload_hex"]
        out = torch.empty_like(xt)
        c.decompress_blocks(out)
        got = out.cpu().numpy().view(np.uint16).ravel()
        if "xhat_bits_prefix" in cs:
            assert [f"{v:04x}" for v in got[: len(cs["xhat_bits_prefix"])]] == cs["xhat_bits_prefix"]
        if cs["scale_bits"] == "3f800000":
            assert np.array_equal(got, x)


def _special_pages(N, d, rng):
    """Pages built to hit every branch: every packet code in both nibbles, RAW triggers, zeros,
    subnormals, the largest finite value, misaligned bodies after run packets."""
    E = N * d
    pages = []
    z = np.zeros((N, d), np.float16)
    pages.append(z.copy())                                                      # all zero
    p = z.copy(); p[0, 0] = -0.0; pages.append(p)                               # -0 only
    p = (rng.standard_normal((N, d)) * 1e-6).astype(np.float16); pages.append(p)  # FP16 subnormals
    p = z.copy(); p[:] = 6e-8; pages.append(p)                                  # smallest subnormal everywhere
    p = rng.standard_normal((N, d)).astype(np.float16); p[N // 2, d // 2] = 65504; pages.append(p)
    p = rng.standard_normal((N, d)).astype(np.float16); p[0, 1] = -65504; pages.append(p)
    for poison in (0x7C00, 0xFC00, 0x7E00, 0xFFFF, 0x7C01):
        p = rng.standard_normal((N, d)).astype(np.float16).view(np.uint16); p[N - 1, d - 1] = poison
        pages.append(p.view(np.float16))
    # integer pages with amax = 127 (s = 1): codes are the values themselves
    p = z.copy(); p[:] = 127; pages.append(p)                                   # one literal + zero runs per row
    p = z.copy(); p[:] = np.arange(d) % 120; p[0, 0] = 127; pages.append(p)     # slope 1: run packets (code 9)
    p = z.copy(); p[:] = -127 + (np.arange(d) * 3) % 250; pages.append(p)       # run packets, wrap-around deltas
    p = z.copy(); p[:, ::2] = 127; p[:, 1::2] = -127; pages.append(p)           # |delta| = 254 -> wraps to +-2
    for w in range(1, 8):                                                       # literal widths 1..7
        p = z.copy()
        p[:] = np.cumsum(rng.integers(-(1 << w) // 4, (1 << w) // 4 + 1, (N, d)), axis=1).clip(-100, 100)
        p[0, 0] = 127
        pages.append(p)
    p = z.copy(); p[:, : d // 2] = np.arange(d // 2) * 2; p[:, d // 2:] = rng.integers(-5, 6, (N, d - d // 2)); p[0, 0] = 127
    pages.append(p)                                                             # run packets then literals: odd body offsets
    p = z.copy(); p[::2] = 64; p[1::2, 3] = 127; pages.append(p)
    p = (rng.standard_normal((N, d)) * np.exp(2 * rng.standard_normal(d))).astype(np.float16); pages.append(p)
    p = rng.standard_normal((N, d)).astype(np.float16); pages.append(p)         # i.i.d.: INT8 fallback
    p = rng.standard_normal((N, d)).astype(np.float16); p[:, 5] *= 100; pages.append(p)
    return np.stack([np.asarray(q, np.float16) for q in pages])


@pytest.mark.parametrize("N,d", [(16, 128), (16, 64), (16, 32), (16, 256), (1, 64), (3, 32), (5, 128), (32, 128),
                                 (16, 96), (16, 160), (16, 192), (16, 224), (8, 96), (5, 224), (32, 96), (1, 96)])
@pytest.mark.parametrize("scheme", [3, 2, 4])
def test_special_pages_all_geometries(N, d, scheme):
    rng = np.random.default_rng(100 + N + d)
    x = _special_pages(N, d, rng)
    n = x.shape[0]
    od = _roundtrip_case(x, N, d, 1, scheme, f"special N={N} d={d}")
    assert (od["mode"][5 + 1:5 + 6] == 0).all()  # the five poisoned pages are stored raw
    if scheme == 3 and N * d >= 1024:
        pool_codes = set()
        _, op = o.compress_pages(x.view(np.uint16), N, d, 3)
        for p in range(n):
            if od["mode"][p] == 3:
                pl = o.page_payload(op, od[p])
                G = N * d // 32
                pool_codes |= {(pl[g >> 1] >> 4) if g & 1 else (pl[g >> 1] & 15) for g in range(G)}
        assert pool_codes >= set(range(0, 10)), pool_codes


@pytest.mark.parametrize("d", [64, 128, 256])
def test_special_pages_channel_pair_mode(d):
    """Mode 5 (channel-pair groups; the GPU builds it for 16-token pages of 64, 128 or 256 channels): every
    branch page, and the geometries it is not built for are refused on the host."""
    rng = np.random.default_rng(777 + d)
    x = _special_pages(16, d, rng)
    # pages for what the mode is about: channel pairs that are zero, constant, narrow and wide
    p = np.zeros((16, d), np.float16); p[:, 6:8] = 3; p[0, 0] = 127; p[:, 20] = np.arange(16) - 8; p[:, d - 2:] = -5
    q = (rng.standard_normal((16, d)) * np.exp(1.5 * rng.standard_normal(d))).astype(np.float16)
    x = np.concatenate([x, p[None], q[None]])
    od = _roundtrip_case(x, 16, d, 1, 5, f"special N=16 d={d} channel pairs")
    assert (od["mode"][5 + 1:5 + 6] == 0).all() and (od["mode"] == 5).sum() > 10
    codes = set()
    _, op = o.compress_pages(x.view(np.uint16), 16, d, 5)
    for i in range(x.shape[0]):
        if od["mode"][i] == 5:
            pl = o.page_payload(op, od[i])
            codes |= {(pl[g >> 1] >> 4) if g & 1 else (pl[g >> 1] & 15) for g in range(d // 2)}
    assert codes >= set(range(0, 10)), codes
    for N, d in ((16, 96), (8, 128), (16, 32), (8, 256)):
        with pytest.raises(kvc.KvcError) as e:
            kvc.Codec(N, d, 1, 5)
        assert e.value.code == kvc.ERR_UNSUPPORTED
        c = kvc.Codec(N, d, 1, 3)
        with pytest.raises(kvc.KvcError) as e:
            c.set_scheme(5)
        assert e.value.code == kvc.ERR_UNSUPPORTED
    # a mode-5 page met by a decoder of another geometry is contained like any unknown mode
    x64 = (rng.standard_normal((3, 16, 96)) * np.exp(rng.standard_normal(96))).astype(np.float16)
    od64, op64 = o.compress_pages(x64.view(np.uint16), 16, 96, 5)
    assert (od64["mode"] == 5).all()
    c = kvc.Codec(16, 96, 1, 3)
    upload_oracle_pool(c, od64, op64)
    out = torch.full((3, 1, 16, 96), 7.0, dtype=torch.float16, device=DEV)
    c.decompress_blocks(out)
    st = c.stats()
    assert st["rc"] == kvc.ERR_CORRUPT and st["status"] & kvc.ST_CORRUPT and bool((out == 0).all())


def test_llama7b_layer_slice_ragged_tail():
    """7B-layer shaped pages (32 heads x 128), a page count that is not a multiple of the
    16-page workgroup batch: 37 blocks x 32 pages."""
    sh = synth.KVShape("7b_slice", 1, 32, 128, 37 * 16, 1)
    x = synth.layer_numpy(sh, 0)  # [2][37][32][16][128]
    for kv, name in ((0, "K"), (1, "V")):
        od = _roundtrip_case(x[kv][:, :31], 16, 128, 31, 3, f"7b-slice {name} ppb=31")
    od = _roundtrip_case(x, 16, 128, 32, 3, "7b-slice K+V")
    assert 2.0 < o.ratio(od, 2048) < 2.6


def test_block_id_indirection_skip_and_reuse():
    rng = np.random.default_rng(7)
    N, d, ppb = 16, 128, 4
    nb = 24
    x = (rng.standard_normal((nb, ppb, N, d)) * np.exp(0.5 * rng.standard_normal(d))).astype(np.float16)
    xt = torch.from_numpy(x).to(DEV)
    c = make_codec(N, d, ppb, 3, n_pool_blocks=40)
    src = np.array([5, 0, -1, 23, 7, 7, 11], np.int32)
    dstp = np.array([30, 2, 9, 0, 39, 17, -1], np.int32)  # pairs with a -1 on either side are skipped
    c.compress_blocks(xt, src_ids=torch.from_numpy(src).to(DEV), pool_ids=torch.from_numpy(dstp).to(DEV))
    st = c.stats()
    assert st["rc"] == 0
    desc = c.desc_numpy().reshape(40, ppb)
    live = [(s, p) for s, p in zip(src, dstp) if s >= 0 and p >= 0]
    assert sum(st["pages"]) == len(live) * ppb and st["pages_invalid"] == (40 - len(live)) * ppb
    pool = c.pool.cpu().numpy()
    for s, p in live:
        for pg in range(ppb):
            dd, pl = o.encode_page(x[s, pg], N, d, 3)
            g = desc[p, pg]
            assert (g["mode"], g["n16"]) == (dd["mode"], dd["n16"]) and g["scale"] == dd["scale"]
            assert pool[int(g["off"]):int(g["off"]) + 16 * int(g["n16"])].tobytes() == pl
    check_pool_invariants(desc.ravel(), st["pool_bytes_used"], pool.size)
    # decode a permuted subset into a larger output, leaving other blocks untouched
    out = torch.full((50, ppb, N, d), 7.0, dtype=torch.float16, device=DEV)
    pids = np.array([39, 2, -1, 30, 0], np.int32)
    dids = np.array([1, 49, 3, -1, 10], np.int32)
    c.decompress_blocks(out, pool_ids=torch.from_numpy(pids).to(DEV), dst_ids=torch.from_numpy(dids).to(DEV))
    got = out.cpu().numpy()
    src_of_pool = {p: s for s, p in live}
    touched = set()
    for p, dd in zip(pids, dids):
        if p < 0 or dd < 0:
            continue
        touched.add(int(dd))
        for pg in range(ppb):
            de, pl = o.encode_page(x[src_of_pool[p], pg], N, d, 3)
            rc, want = o.decode_page(pl, de, N, d)
            assert np.array_equal(got[dd, pg].view(np.uint16).ravel(), want)
    for b in set(range(50)) - touched:
        assert (got[b] == 7.0).all()
    assert c.stats()["status"] == 0


def test_gather_decompress_small_pattern():
    """Translation table + predicted ids (Algorithm 1's fetch) on a 3-layer toy pool, K and V of
    2 heads per block (ppb = 4)."""
    rng = np.random.default_rng(21)
    N, d, ppb, n_layers = 16, 128, 4, 3
    pat = synth.gather_pattern(n_seq=5, k=8, len_lo=40, len_hi=300, seed=3)
    pbl = pat.pool_blocks_per_layer
    x = (rng.standard_normal((n_layers * pbl, ppb, N, d)) * np.exp(0.5 * rng.standard_normal(d))).astype(np.float16)
    c, xt = gpu_compress(x, N, d, ppb, 3)
    od, op = o.compress_pages(x.view(np.uint16), N, d, 3, n_threads=8)
    full, _ = o.decompress_pages(op, od, N, d, n_threads=8)
    full = full.reshape(n_layers, pbl, ppb, N, d)
    table = torch.from_numpy(pat.block_table).to(DEV)
    for step in (0, 1, 999):
        pred_np = pat.predictions(step).copy()
        if step == 1:
            pred_np[2, 3] = -1  # skipped: output block stays as it was
        pred = torch.from_numpy(pred_np).to(DEV)
        out = torch.full((n_layers * pat.n_seq * pat.k, ppb, N, d), 3.0, dtype=torch.float16, device=DEV)
        c.gather_decompress(out, table, pred, n_layers, pbl)
        got = out.cpu().numpy().view(np.uint16).reshape(n_layers, pat.n_seq, pat.k, ppb, N, d)
        for l in range(n_layers):
            for s in range(pat.n_seq):
                for j in range(pat.k):
                    lb = pred_np[s, j]
                    if lb < 0:
                        assert (got[l, s, j].view(np.float16) == 3.0).all()
                    else:
                        assert np.array_equal(got[l, s, j], full[l, pat.block_table[s, lb]]), (step, l, s, j)
    assert c.stats()["status"] == 0
    # out-of-range prediction / table entry: zero-filled + status bit, nothing else disturbed
    pred_np = pat.predictions(5).copy()
    pred_np[0, 0] = pat.max_blocks + 3
    out = torch.full((n_layers * pat.n_seq * pat.k, ppb, N, d), 3.0, dtype=torch.float16, device=DEV)
    c.gather_decompress(out, table, torch.from_numpy(pred_np).to(DEV), n_layers, pbl)
    got = out.cpu().numpy().reshape(n_layers, pat.n_seq, pat.k, -1)
    assert (got[:, 0, 0] == 0).all() and not (got[:, 0, 1] == 0).all()
    st = c.stats()
    assert st["status"] & kvc.ST_BAD_INDEX and st["rc"] == kvc.ERR_CORRUPT


def test_gather_hand_counted_table_entries():
    """Hand-counted fetch through a translation table: two layers of 7 pool blocks, one sequence with table entries
    (6, 7, -1) and predictions (0, 1, 2).  Entry 6 is the layer's last block: layer l reads pool block 7 l + 6.
    Entry 7 equals the layer's block count: a bad index, its output block is zero-filled.  Entry -1: the
    sequence has no such block, its output block is left as it was."""
    rng = np.random.default_rng(31)
    N, d, ppb, n_layers, pbl = 16, 64, 2, 2, 7
    x = rng.standard_normal((n_layers * pbl, ppb, N, d)).astype(np.float16)
    c, _ = gpu_compress(x, N, d, ppb, 3)
    od, op = o.compress_pages(x.view(np.uint16), N, d, 3)
    full = o.decompress_pages(op, od, N, d)[0].reshape(n_layers * pbl, ppb, N, d)
    table = torch.tensor([[6, 7, -1]], dtype=torch.int32, device=DEV)
    pred = torch.tensor([[0, 1, 2]], dtype=torch.int32, device=DEV)
    out = torch.full((n_layers * 3, ppb, N, d), 3.0, dtype=torch.float16, device=DEV)
    c.gather_decompress(out, table, pred, n_layers, pbl)
    got = out.cpu().numpy().view(np.uint16).reshape(n_layers, 3, ppb, N, d)
    for l in range(n_layers):
        assert np.array_equal(got[l, 0], full[7 * l + 6])
        assert not got[l, 1].any()
        assert (got[l, 2].view(np.float16) == 3.0).all()
    st = c.stats()
    assert st["status"] == kvc.ST_BAD_INDEX and st["rc"] == kvc.ERR_CORRUPT


def test_pool_exhaustion_marks_pages_invalid():
    rng = np.random.default_rng(5)
    N, d, ppb = 16, 128, 1
    x = rng.standard_normal((64, ppb, N, d)).astype(np.float16)  # i.i.d.: every page 2048 B (INT8)
    c, xt = gpu_compress(x, N, d, ppb, 3, pool_bytes=20 * 2048 + 512)
    st = c.stats()
    assert st["rc"] == kvc.ERR_POOL_FULL and st["status"] & kvc.ST_POOL_FULL
    desc = c.desc_numpy()
    ok = desc["mode"] != 0xFF
    assert 0 < ok.sum() <= 20 and st["pages_invalid"] == 64 - ok.sum()
    assert ((desc["off"][ok] + 2048) <= 20 * 2048 + 512).all()
    out = torch.full_like(xt, 1.0)
    c.decompress_blocks(out)
    got = out.cpu().numpy().view(np.uint16).reshape(64, N, d)
    for p in range(64):
        if ok[p]:
            dd, pl = o.encode_page(x[p], N, d, 3)
            assert np.array_equal(got[p].ravel(), o.decode_page(pl, dd, N, d)[1])
        else:
            assert not got[p].any()  # undecodable pages are zero-filled
    assert c.stats()["status"] & kvc.ST_CORRUPT
    c.reset_pool()
    st = c.stats()
    assert st["status"] == 0 and st["pool_bytes_used"] == 0 and st["pages_invalid"] == 64


def test_corrupt_descriptors_and_payloads_are_contained():
    rng = np.random.default_rng(6)
    N, d = 16, 128
    x = rng.standard_normal((8, N, d)).astype(np.float16)
    x[:, :, 3] *= 40
    od, op = o.compress_pages(x.view(np.uint16), N, d, 3)
    assert (od["mode"] == 3).all()
    good, _ = o.decompress_pages(op, od, N, d)
    bd = od.copy()
    bp = op.copy()
    bd[0]["mode"] = 9                      # unknown mode
    bd[1]["off"] = op.size + 4096          # span outside the pool
    bd[2]["n16"] = bd[2]["n16"] - 1        # truncated payload
    bd[3]["off"] += 8                      # misaligned
    bp[int(od[4]["off"])] = 0xAB           # header codes 11 and 10
    bd[5]["mode"] = 1                      # wrong size for INT8
    c = kvc.Codec(N, d, 1, 3)
    upload_oracle_pool(c, bd, bp)
    out = torch.full((8, 1, N, d), 2.0, dtype=torch.float16, device=DEV)
    c.decompress_blocks(out)
    got = out.cpu().numpy().view(np.uint16).reshape(8, N, d)
    want, nbad = o.decompress_pages(bp, bd, N, d)
    assert nbad == 6
    assert np.array_equal(got, want)
    assert not got[:6].any() and np.array_equal(got[6:], good[6:])
    st = c.stats()
    assert st["status"] & kvc.ST_CORRUPT and st["rc"] == kvc.ERR_CORRUPT


def test_hand_built_payloads_decode_or_are_refused_on_gpu():
    """The payloads typed in by hand that pin the oracle's decoder (tests/handbuilt_payloads.py), through the GPU
    decoder: packet codes, the codes a mode admits, exact payload size, the bound below the INT8 size."""
    import handbuilt_payloads as hb

    desc = np.zeros(len(hb.CASES), o.DESC_DTYPE)
    chunks, off = [], 0
    for i, (name, mode, payload, ok, values) in enumerate(hb.CASES):
        desc[i]["off"], desc[i]["scale"], desc[i]["n16"], desc[i]["mode"] = off, hb.SCALE, len(payload) // 16, mode
        chunks.append(np.frombuffer(payload, np.uint8))
        off += len(payload)
    pool = np.concatenate(chunks)
    c = kvc.Codec(hb.N, hb.D, 1, 3)
    upload_oracle_pool(c, desc, pool)
    out = torch.full((len(hb.CASES), 1, hb.N, hb.D), 2.0, dtype=torch.float16, device=DEV)
    c.decompress_blocks(out)
    got = out.cpu().numpy().view(np.uint16).reshape(len(hb.CASES), hb.N, hb.D)
    want, nbad = o.decompress_pages(pool, desc, hb.N, hb.D)
    assert np.array_equal(got, want.reshape(got.shape)) and nbad == sum(not ok for _, _, _, ok, _ in hb.CASES)
    for i, (name, mode, payload, ok, values) in enumerate(hb.CASES):
        if ok:
            assert np.array_equal(got[i], values.view(np.uint16)), name
        else:
            assert not got[i].any(), name
    st = c.stats()
    assert st["status"] & kvc.ST_CORRUPT and st["rc"] == kvc.ERR_CORRUPT


def test_products_next_to_a_tie_on_gpu():
    """Pages whose elements multiply with s^-1 to a hair beside k + 1/2 (tests/adversarial_inputs.py, the inputs
    of the oracle's pin): one page per page maximum, holding that maximum and every such element with both signs.
    Codes compared through the INT8 scheme (the codes themselves) and the full scheme."""
    import adversarial_inputs as adv

    by_amax = {}
    for amax, xv, q in adv.near_half_products():
        by_amax.setdefault(float(amax), []).append((xv, q))
    N, d = 16, 128
    x = np.zeros((len(by_amax), N * d), np.float16)
    want_q = np.zeros((len(by_amax), N * d), np.int8)
    for i, (amax, lst) in enumerate(sorted(by_amax.items())):
        x[i, 0], want_q[i, 0] = amax, 127
        for j, (xv, q) in enumerate(lst):
            x[i, 1 + 2 * j], x[i, 2 + 2 * j] = xv, -xv
            want_q[i, 1 + 2 * j], want_q[i, 2 + 2 * j] = q, -q
    x = x.reshape(-1, N, d)
    for scheme in (1, 3):
        c, _ = gpu_compress(x, N, d, 1, scheme)
        desc, pool = c.desc_numpy(), c.pool.cpu().numpy()
        compare_pages_with_oracle(x.view(np.uint16), desc, pool, N, d, scheme)
        if scheme == 1:  # the payload is the codes: compare with the exact-arithmetic values directly
            assert (desc["mode"] == 1).all()
            got = np.stack([pool[int(o_):int(o_) + N * d] for o_ in desc["off"]]).view(np.int8)
            assert np.array_equal(got, want_q)


def test_host_side_argument_errors():
    c = kvc.Codec(16, 128, 2, 3)
    x = torch.zeros((4, 2, 16, 128), dtype=torch.float16, device=DEV)
    with pytest.raises(kvc.KvcError) as e:
        c.compress_blocks(x)
    assert e.value.code == kvc.ERR_NOT_BOUND
    c.alloc_pool(2, 1 << 16, DEV)
    with pytest.raises(kvc.KvcError) as e:
        c.compress_blocks(x)  # 4 blocks, 2 pool blocks, identity ids
    assert e.value.code == kvc.ERR_ARG
    with pytest.raises(kvc.KvcError) as e:
        kvc.Codec(16, 288, 1, 3)
    assert e.value.code == kvc.ERR_UNSUPPORTED
    with pytest.raises(kvc.KvcError) as e:
        kvc.Codec(16, 100, 1, 3)
    assert e.value.code == kvc.ERR_ARG
    c.compress_blocks(x, n=0)
    assert c.stats()["pages_invalid"] == 4
    # one call handles at most 2^26 - 4 pages: beyond that the host refuses before anything is launched
    # (the counts below are only numbers to the host checks; no buffer of that size exists or is touched)
    L = kvc.load()
    big = kvc.Codec(16, 128, 4, 3)
    assert L.kvc_bind_pool(big._ctx, c.pool.data_ptr(), c.pool.numel(), c.desc.data_ptr(), 1 << 27) == kvc.OK
    n_over = (1 << 24)  # blocks of 4 pages: 2^26 pages
    assert L.kvc_compress_blocks(big._ctx, x.data_ptr(), n_over, None, None, n_over, None) == kvc.ERR_ARG
    assert L.kvc_decompress_blocks(big._ctx, x.data_ptr(), n_over, None, None, n_over, None) == kvc.ERR_ARG
    assert L.kvc_copy_bytes(x.data_ptr(), x.data_ptr(), (1 << 38) - 4096 + 16, None) == kvc.ERR_ARG


def test_per_block_scheme_selection():
    """kvc_compress_blocks_mixed: the requested mode is a per-block argument (layer-wise selection)."""
    rng = np.random.default_rng(44)
    N, d, ppb, nb = 16, 128, 4, 40
    x = (rng.standard_normal((nb, ppb, N, d)) * np.exp(0.7 * rng.standard_normal(d))).astype(np.float16)
    schemes = rng.integers(0, 6, nb).astype(np.uint8)
    schemes[:6] = [0, 1, 2, 3, 4, 5]
    xt = torch.from_numpy(x).to(DEV)
    c = make_codec(N, d, ppb, 3, nb, pool_bytes=nb * ppb * N * d * 2 + 64)
    c.compress_blocks(xt, block_scheme=torch.from_numpy(schemes).to(DEV))
    st = c.stats()
    assert st["rc"] == 0
    desc = c.desc_numpy().reshape(nb, ppb)
    pool = c.pool.cpu().numpy()
    for b in range(nb):
        for pg in range(ppb):
            dd, pl = o.encode_page(x[b, pg], N, d, int(schemes[b]))
            g = desc[b, pg]
            assert (g["mode"], g["n16"]) == (dd["mode"], dd["n16"]) and g["scale"] == dd["scale"], (b, pg, schemes[b])
            assert pool[int(g["off"]):int(g["off"]) + 16 * int(g["n16"])].tobytes() == pl
    check_pool_invariants(desc.ravel(), st["pool_bytes_used"], pool.size)
    out = torch.empty_like(xt)
    c.decompress_blocks(out)
    got = out.cpu().numpy().view(np.uint16)
    for b in range(nb):
        for pg in range(ppb):
            dd, pl = o.encode_page(x[b, pg], N, d, int(schemes[b]))
            assert np.array_equal(got[b, pg].ravel(), o.decode_page(pl, dd, N, d)[1])
    assert (got[schemes == 0] == x.view(np.uint16)[schemes == 0]).all()  # RAW blocks come back bit-exact


@pytest.mark.parametrize("N,d,highest", [(16, 128, 5), (16, 64, 5), (16, 96, 4), (8, 128, 4)])
def test_per_block_modes_above_the_highest_are_read_as_the_highest(N, d, highest):
    """kvc_compress_blocks_mixed documents that a requested mode above the highest the page shape has (5 where
    mode 5 exists, else 4) is read as that highest mode."""
    rng = np.random.default_rng(46 + d)
    nb = 12
    x = (rng.standard_normal((nb, 1, N, d)) * np.exp(0.7 * rng.standard_normal(d))).astype(np.float16)
    asked = np.array([highest, highest + 1, 6, 7, 9, 100, 128, 200, 254, 255, 3, 0], np.uint8)
    c = make_codec(N, d, 1, 3, nb)
    c.compress_blocks(torch.from_numpy(x).to(DEV), block_scheme=torch.from_numpy(asked).to(DEV))
    assert c.stats()["rc"] == 0
    desc, pool = c.desc_numpy(), c.pool.cpu().numpy()
    for b in range(nb):
        dd, pl = o.encode_page(x[b, 0], N, d, min(int(asked[b]), highest))
        g = desc[b]
        assert (g["mode"], g["n16"]) == (dd["mode"], dd["n16"]) and g["scale"] == dd["scale"], (b, asked[b])
        assert pool[int(g["off"]):int(g["off"]) + 16 * int(g["n16"])].tobytes() == pl


def test_pool_in_pinned_host_memory():
    """The compressed pool behind the host link (slow-tier emulation): same bytes as the oracle, read
    straight from the pinned buffer on the CPU; pageable memory is refused."""
    rng = np.random.default_rng(55)
    N, d, ppb, nb = 16, 128, 2, 24
    x = (rng.standard_normal((nb, ppb, N, d)) * np.exp(0.6 * rng.standard_normal(d))).astype(np.float16)
    xt = torch.from_numpy(x).to(DEV)
    c = kvc.Codec(N, d, ppb, 3)
    pool, desc = c.alloc_pool(nb, nb * ppb * N * d + 64, DEV, host_pool=True)
    assert not pool.is_cuda and pool.is_pinned()
    c.compress_blocks(xt)
    out = torch.empty_like(xt)
    c.decompress_blocks(out)
    st = c.stats()  # synchronises
    assert st["rc"] == 0
    compare_pages_with_oracle(x.view(np.uint16).reshape(-1, N, d), c.desc_numpy(), pool.numpy(), N, d, 3)
    od, op = o.compress_pages(x.view(np.uint16), N, d, 3)
    assert np.array_equal(out.cpu().numpy().view(np.uint16).reshape(-1, N, d), o.decompress_pages(op, od, N, d)[0])
    c2 = kvc.Codec(N, d, ppb, 3)
    pageable = torch.empty(4096, dtype=torch.uint8)
    rc = kvc.load().kvc_bind_pool(c2._ctx, pageable.data_ptr(), 4096, desc.data_ptr(), 4)
    assert rc == kvc.ERR_ARG
    # the refused call leaves no HIP error behind: the next launches of either context report their own status
    c.reset_pool()
    c.compress_blocks(xt)
    assert c.stats()["rc"] == 0


@pytest.mark.parametrize("d,H,pad", [(128, 4, 0), (128, 3, 64), (64, 2, 8), (256, 2, 0)])
def test_strided_cache_layout(d, H, pad):
    """Token-major cache [block][token][head][d (+pad)]: pages are strided views, no copy is made.
    Compress reads the view, decompress / gather write the view and leave the padding alone."""
    rng = np.random.default_rng(60 + d + H)
    N, nb = 16, 21
    row = H * d + pad
    x = (rng.standard_normal((nb, N, row)) * 1.5).astype(np.float16)
    x[..., : H * d] *= np.exp(0.5 * rng.standard_normal(H * d)).astype(np.float16)
    x[2, 3, 5] = np.float16("inf")  # one RAW page, through the strided copy path
    pages = np.stack([x[:, :, h * d:(h + 1) * d] for h in range(H)], axis=1)  # dense [nb][H][N][d]
    xt = torch.from_numpy(x).to(DEV)
    c = kvc.Codec(N, d, H, 3)
    c.set_cache_layout(block_stride=N * row, page_stride=d, row_stride=row)
    c.alloc_pool(nb, nb * H * N * d * 2 + 64, DEV)
    c.compress_blocks(xt)
    st = c.stats()
    assert st["rc"] == 0 and sum(st["pages"]) == nb * H and st["pages"][0] == 1
    od, op = compare_pages_with_oracle(np.ascontiguousarray(pages).view(np.uint16).reshape(-1, N, d), c.desc_numpy(),
                                       c.pool.cpu().numpy(), N, d, 3)
    want, _ = o.decompress_pages(op, od, N, d)
    want = want.reshape(nb, H, N, d)
    out = torch.full((nb + 2, N, row), 7.0, dtype=torch.float16, device=DEV)
    dst = torch.from_numpy(rng.permutation(nb + 2)[:nb].astype(np.int32)).to(DEV)
    c.decompress_blocks(out, n=nb, dst_ids=dst)
    got = out.cpu().numpy()
    dst_np = dst.cpu().numpy()
    for b in range(nb):
        for h in range(H):
            assert np.array_equal(got[dst_np[b], :, h * d:(h + 1) * d].view(np.uint16), want[b, h]), (b, h)
    if pad:
        assert (got[..., H * d:] == 7.0).all()
    untouched = sorted(set(range(nb + 2)) - set(dst_np.tolist()))
    assert (got[untouched] == 7.0).all()
    assert c.stats()["status"] == 0
    with pytest.raises(kvc.KvcError):
        c.set_cache_layout(block_stride=N * row, page_stride=d, row_stride=d - 8)
    with pytest.raises(kvc.KvcError):
        c.set_cache_layout(block_stride=N * row + 4, page_stride=d, row_stride=row)


@pytest.mark.parametrize("nbytes", [16, 4096 - 16, 4096, 4096 + 16, 3 * 16384 + 48, (1 << 20) + 4080])
def test_copy_yardstick_copies_every_byte(nbytes):
    """The bandwidth yardstick is a real copy: ragged sizes around its 4 KB and 16 KB work units, nothing
    written past the end."""
    g = torch.Generator(device="cpu").manual_seed(nbytes)
    src = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, generator=g).to(DEV)
    buf = torch.full((nbytes + 64,), 0xA5, dtype=torch.uint8, device=DEV)
    kvc.copy_bytes(buf[:nbytes], src)
    torch.cuda.synchronize()
    assert torch.equal(buf[:nbytes], src) and bool((buf[nbytes:] == 0xA5).all())


def test_device_clocks_hook():
    ck = kvc.device_clocks()
    assert ck["shader_khz"] > 100_000 and ck["memory_khz"] > 100_000 and ck["memory_bus_bits"] >= 1024, ck
    assert kvc.load().kvc_device_clocks(None, None, None) == kvc.OK


def test_pool_checkpoint_and_resume():
    """Pool bytes, descriptor table and the used-byte count are a complete checkpoint: restored into fresh
    buffers of another context, the saved pages decode as before and compression goes on behind them."""
    N, d, ppb, scheme = 16, 128, 2, 3
    rng = np.random.default_rng(2024)
    x = (rng.standard_normal((600, ppb, N, d)) * np.exp(0.5 * rng.standard_normal(d))).astype(np.float16)
    x[17] = 0
    xt = torch.from_numpy(x).to(DEV)
    a = kvc.Codec(N, d, ppb, scheme)
    a.alloc_pool(600, 600 * ppb * N * d * 2 + 64, DEV)
    a.compress_blocks(xt[:350], n=350)  # pool blocks 0..349
    st = a.stats()
    assert st["rc"] == 0
    used = st["pool_bytes_used"]
    saved_pool, saved_desc = a.pool.cpu(), a.desc.cpu()
    del a
    b = kvc.Codec(N, d, ppb, scheme)
    b.bind_pool(saved_pool.to(DEV), saved_desc.to(DEV))
    with pytest.raises(kvc.KvcError) as e:
        b.restore_pool(used + 8)  # not a multiple of 16
    assert e.value.code == kvc.ERR_ARG
    with pytest.raises(kvc.KvcError) as e:
        b.restore_pool(saved_pool.numel() + 16)  # beyond the pool
    assert e.value.code == kvc.ERR_ARG
    b.restore_pool(used)
    ids = torch.arange(350, 600, dtype=torch.int32, device=DEV)
    b.compress_blocks(xt, src_ids=ids, pool_ids=ids)  # the rest, behind the restored payloads
    out = torch.empty_like(xt)
    b.decompress_blocks(out)
    st = b.stats()
    assert st["rc"] == 0 and st["pool_bytes_used"] > used
    desc, pool = b.desc_numpy(), b.pool.cpu().numpy()
    check_pool_invariants(desc, st["pool_bytes_used"], pool.size)
    od, op = compare_pages_with_oracle(x.reshape(-1, N, d).view(np.uint16), desc, pool, N, d, scheme)
    want, bad = o.decompress_pages(op, od, N, d, n_threads=8)
    assert bad == 0 and np.array_equal(out.cpu().numpy().view(np.uint16).reshape(-1, N, d), want)
    assert np.array_equal(pool[:used], saved_pool.numpy()[:used]), "the restored payloads were not touched"
