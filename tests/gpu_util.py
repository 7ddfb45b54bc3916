"""Helpers for the GPU parity tests: run the HIP library on numpy inputs and compare page by page
with the CPU oracle.  Placement of payloads inside the pool is free, so pages are compared through
their descriptors; `off` is checked by invariants only."""
import numpy as np
import torch

from oracle import kvc_oracle as o
from paper_2512_11920_amd import kvc

DEV = "cuda:0"


def make_codec(N, d, ppb, scheme, n_pool_blocks, pool_bytes=None):
    c = kvc.Codec(N, d, ppb, scheme)
    if pool_bytes is None:
        pool_bytes = n_pool_blocks * ppb * N * d * 2 + 64
    c.alloc_pool(n_pool_blocks, pool_bytes, DEV)
    return c


def gpu_compress(x: np.ndarray, N, d, ppb, scheme, **kw):
    """x: float16/uint16 [..., N, d] with a whole number of blocks.  -> (codec, cache tensor)."""
    xt = torch.from_numpy(np.require(x, requirements=["C", "W"]).view(np.float16).reshape(-1, ppb, N, d)).to(DEV)
    c = make_codec(N, d, ppb, scheme, xt.shape[0], **kw)
    c.compress_blocks(xt)
    torch.cuda.synchronize()
    return c, xt


def check_pool_invariants(desc: np.ndarray, pool_bytes_used: int, pool_bytes: int):
    live = desc[desc["mode"] != 0xFF]
    off = live["off"].astype(np.int64)
    size = live["n16"].astype(np.int64) * 16
    assert (off % 16 == 0).all()
    assert (off + size <= pool_bytes).all()
    order = np.argsort(off, kind="stable")
    assert (off[order][1:] >= (off + size)[order][:-1]).all(), "payload spans overlap"
    assert int(size.sum()) == pool_bytes_used
    if live.size:
        assert off.min() == 0 and int((off + size).max()) == pool_bytes_used, "spans do not tile [0, used)"


def compare_pages_with_oracle(x_pages_u16: np.ndarray, desc: np.ndarray, pool: np.ndarray, N, d, scheme):
    """Bit-exact comparison of every page: mode, n16, scale bits, payload bytes incl. padding."""
    n = x_pages_u16.shape[0]
    od, op = o.compress_pages(x_pages_u16, N, d, scheme, n_threads=8)
    assert desc.shape[0] == n
    assert np.array_equal(desc["mode"], od["mode"]), np.nonzero(desc["mode"] != od["mode"])[0][:10]
    assert np.array_equal(desc["n16"], od["n16"]), np.nonzero(desc["n16"] != od["n16"])[0][:10]
    assert np.array_equal(desc["scale"].view(np.uint32), od["scale"].view(np.uint32))
    assert not desc["rsvd"].any()
    # payload bytes: gather both sides into page order and compare in one shot
    size = od["n16"].astype(np.int64) * 16
    idx_g = np.repeat(desc["off"].astype(np.int64) - np.concatenate([[0], np.cumsum(size)[:-1]]), size) + np.arange(size.sum())
    got = pool[idx_g]
    if not np.array_equal(got, op):
        bad = np.nonzero(got != op)[0][0]
        page = int(np.searchsorted(np.cumsum(size), bad, side="right"))
        raise AssertionError(f"payload differs first at page {page} (mode {od['mode'][page]}), byte {bad - (np.cumsum(size)[page] - size[page])}")
    return od, op


def upload_oracle_pool(codec, od: np.ndarray, op: np.ndarray):
    """Bind a pool/descriptor table produced by the oracle to a codec (decode-side tests)."""
    pool = torch.zeros(max(16, (op.size + 15) // 16 * 16), dtype=torch.uint8, device=DEV)
    pool[: op.size] = torch.from_numpy(op).to(DEV)
    desc = torch.from_numpy(od.view(np.uint8).copy()).to(DEV)
    codec.bind_pool(pool, desc)
    return pool, desc


def fetch_pages(codec, page_ids: np.ndarray):
    """Descriptors and payload bytes of the given descriptor-table entries, compacted on the GPU and
    copied to the host: -> (desc records with `off` rewritten to the compact buffer, uint8 buffer)."""
    idt = torch.from_numpy(np.ascontiguousarray(page_ids, np.int64)).to(codec.desc.device)
    d = codec.desc.view(-1, 16)[idt].cpu().numpy().view(kvc.DESC_DTYPE).ravel().copy()
    live = d["mode"] != 0xFF
    size = np.where(live, d["n16"].astype(np.int64) * 16, 0)
    start = np.concatenate([[0], np.cumsum(size)[:-1]])
    total = int(size.sum())
    shift = torch.from_numpy(d["off"].astype(np.int64) - start).to(idt.device)
    idx = torch.repeat_interleave(shift, torch.from_numpy(size).to(idt.device)) + torch.arange(total, device=idt.device)
    buf = codec.pool[idx].cpu().numpy()
    d["off"] = start.astype(np.uint64)
    return d, buf
