"""ctypes access to the CPU oracle (oracle/kvc_oracle.c).

TEST INFRASTRUCTURE: only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this module.  The GPU package never does.

The C file is the oracle; this module only builds it with gcc, marshals numpy arrays in and
out, and adds the two bookkeeping formulas that are sums over descriptors (compression ratio
R_c of Section 3.5.2 and the per-page size closed form).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# The two paths can be redirected so that tests/test_oracle_mutations.py can build copies of the C file with a
# mistake planted in them and show that the pins notice; nothing else sets these variables.
_SRC = os.environ.get("KVC_ORACLE_SRC") or os.path.join(_HERE, "kvc_oracle.c")
_LIB = os.environ.get("KVC_ORACLE_LIB") or os.path.join(_HERE, "libkvc_oracle.so")

MODE_RAW, MODE_INT8, MODE_DELTA, MODE_RLE, MODE_PACK, MODE_CHAN, MODE_INVALID = 0, 1, 2, 3, 4, 5, 0xFF

#: numpy view of the 16-byte page descriptor (little-endian, no padding)
DESC_DTYPE = np.dtype(
    [("off", "<u8"), ("scale", "<f4"), ("n16", "<u2"), ("mode", "u1"), ("rsvd", "u1")]
)
assert DESC_DTYPE.itemsize == 16


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
               "-pthread", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        u16p, u8p, i8p = C.POINTER(C.c_uint16), C.POINTER(C.c_uint8), C.POINTER(C.c_int8)
        L.kvo_half_to_float.restype = C.c_float
        L.kvo_half_to_float.argtypes = [C.c_uint16]
        L.kvo_float_to_half.restype = C.c_uint16
        L.kvo_float_to_half.argtypes = [C.c_float]
        L.kvo_quantize_page.restype = C.c_int
        L.kvo_quantize_page.argtypes = [u16p, C.c_int, C.POINTER(C.c_float), C.POINTER(C.c_float), i8p]
        L.kvo_delta_zigzag.restype = None
        L.kvo_delta_zigzag.argtypes = [i8p, C.c_int, C.c_int, u8p]
        L.kvo_rle_pack.restype = C.c_size_t
        L.kvo_rle_pack.argtypes = [u8p, C.c_int, C.c_int, u8p]
        L.kvo_encode_page.restype = C.c_int64
        L.kvo_encode_page.argtypes = [u16p, C.c_int, C.c_int, C.c_int, u8p, C.c_void_p]
        L.kvo_decode_codes.restype = C.c_int
        L.kvo_decode_codes.argtypes = [u8p, C.c_size_t, C.c_int, C.c_int, C.c_int, i8p]
        L.kvo_decode_page.restype = C.c_int
        L.kvo_decode_page.argtypes = [u8p, C.c_void_p, C.c_int, C.c_int, u16p]
        L.kvo_compress_pages.restype = C.c_int64
        L.kvo_compress_pages.argtypes = [u16p, C.c_int64, C.c_int, C.c_int, C.c_int, u8p, C.c_uint64,
                                         C.c_void_p, C.c_int]
        L.kvo_decompress_pages.restype = C.c_int64
        L.kvo_decompress_pages.argtypes = [u8p, C.c_uint64, C.c_void_p, C.POINTER(C.c_int64), C.c_int64,
                                           C.c_int, C.c_int, u16p, C.c_int]
        _lib = L
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def _as_u16(x) -> np.ndarray:
    x = np.asarray(x)
    if x.dtype == np.float16:
        x = x.view(np.uint16)
    assert x.dtype == np.uint16, x.dtype
    return np.ascontiguousarray(x)


def half_to_float(bits: int) -> float:
    return float(lib().kvo_half_to_float(int(bits)))


def float_to_half(v: float) -> int:
    return int(lib().kvo_float_to_half(C.c_float(v)))


def quantize_page(x):
    """Scaling + quantize steps of Alg. 2 on one page.  -> (nonfinite, s, s_inv, q[int8])."""
    x = _as_u16(x).ravel()
    s, si = C.c_float(0), C.c_float(0)
    q = np.zeros(x.size, np.int8)
    nf = lib().kvo_quantize_page(_p(x, C.c_uint16), x.size, C.byref(s), C.byref(si), _p(q, C.c_int8))
    return bool(nf), np.float32(s.value), np.float32(si.value), q


def delta_zigzag(q, N: int, d: int) -> np.ndarray:
    q = np.ascontiguousarray(q, np.int8).ravel()
    assert q.size == N * d
    u = np.zeros(N * d, np.uint8)
    lib().kvo_delta_zigzag(_p(q, C.c_int8), N, d, _p(u, C.c_uint8))
    return u


def rle_pack(u, with_runs: bool = True) -> bytes:
    u = np.ascontiguousarray(u, np.uint8).ravel()
    out = np.zeros(u.size + u.size // 64 + 1, np.uint8)
    n = lib().kvo_rle_pack(_p(u, C.c_uint8), u.size, int(with_runs), _p(out, C.c_uint8))
    return out[:n].tobytes()


def encode_page(x, N: int, d: int, scheme: int = MODE_RLE):
    """One page -> (descriptor record, payload bytes incl. zero padding)."""
    x = _as_u16(x).ravel()
    assert x.size == N * d
    desc = np.zeros(1, DESC_DTYPE)
    payload = np.zeros(2 * N * d, np.uint8)
    n = lib().kvo_encode_page(_p(x, C.c_uint16), N, d, scheme, _p(payload, C.c_uint8), desc.ctypes.data)
    if n < 0:
        raise ValueError(f"kvo_encode_page error {n}")
    return desc[0], payload[:n].tobytes()


def decode_codes(payload: bytes, mode: int, N: int, d: int):
    buf = np.frombuffer(payload, np.uint8).copy()
    q = np.zeros(N * d, np.int8)
    rc = lib().kvo_decode_codes(_p(buf, C.c_uint8), buf.size, mode, N, d, _p(q, C.c_int8))
    return rc, q


def decode_page(payload: bytes, desc, N: int, d: int):
    """-> (rc, uint16[N*d] FP16 bit patterns)."""
    buf = np.frombuffer(payload, np.uint8).copy()
    if buf.size == 0:
        buf = np.zeros(1, np.uint8)
    dd = np.zeros(1, DESC_DTYPE)
    dd[0] = desc
    out = np.full(N * d, 0xFFFF, np.uint16)  # the C side writes every element: values, or zeros for a refused page
    rc = lib().kvo_decode_page(_p(buf, C.c_uint8), dd.ctypes.data, N, d, _p(out, C.c_uint16))
    return rc, out


def compress_pages(x, N: int, d: int, scheme: int = MODE_RLE, n_threads: int = 1):
    """x: [..., N, d] FP16 (or uint16 bits).  -> (desc[n_pages], pool uint8[used])."""
    x = _as_u16(x)
    E = N * d
    assert x.size % E == 0
    n_pages = x.size // E
    cap = n_pages * E * 2 + 16
    pool = np.empty(cap, np.uint8)
    desc = np.zeros(n_pages, DESC_DTYPE)
    used = lib().kvo_compress_pages(_p(x, C.c_uint16), n_pages, N, d, scheme, _p(pool, C.c_uint8), cap,
                                    desc.ctypes.data, n_threads)
    if used < 0:
        raise ValueError(f"kvo_compress_pages error {used}")
    return desc, pool[:used]


def decompress_pages(pool, desc, N: int, d: int, page_ids=None, n_threads: int = 1):
    """-> (uint16[n_pages, N, d], number of undecodable pages)."""
    pool = np.ascontiguousarray(pool, np.uint8)
    desc = np.ascontiguousarray(desc, DESC_DTYPE)
    if page_ids is None:
        n_pages, ids_p = desc.size, None
    else:
        page_ids = np.ascontiguousarray(page_ids, np.int64)
        n_pages, ids_p = page_ids.size, _p(page_ids, C.c_int64)
    out = np.full((n_pages, N, d), 0xFFFF, np.uint16)  # as in decode_page
    pool_arg = pool if pool.size else np.zeros(16, np.uint8)
    bad = lib().kvo_decompress_pages(_p(pool_arg, C.c_uint8), pool.size, desc.ctypes.data, ids_p, n_pages, N, d,
                                     _p(out, C.c_uint16), n_threads)
    return out, int(bad)


def page_payload(pool, d) -> bytes:
    """Payload bytes (padding included) of one descriptor record."""
    o, n = int(d["off"]), int(d["n16"]) * 16
    return bytes(memoryview(np.ascontiguousarray(pool, np.uint8))[o:o + n])


def ratio(desc, E: int) -> float:
    """R_c = uncompressed bytes / (payload bytes + 16-byte descriptors)  (Section 3.5.2)."""
    desc = np.asarray(desc)
    return float(desc.size * E * 2) / float(desc["n16"].astype(np.int64).sum() * 16 + 16 * desc.size)
