"""Thin ctypes binding of libkvc.so (see include/kvc.h).  Argument marshalling only: every step
of the codec runs in the HIP kernels.  PyTorch supplies device memory and streams.

There is no CPU fallback: if the library has not been built (``python -m paper_2512_11920_amd.build``)
loading raises."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libkvc.so")

OK, ERR_ARG, ERR_NOT_BOUND, ERR_HIP, ERR_POOL_FULL, ERR_CORRUPT, ERR_UNSUPPORTED, ERR_TOO_LARGE = 0, -1, -2, -3, -4, -5, -6, -7
MODE_RAW, MODE_INT8, MODE_DELTA, MODE_RLE, MODE_PACK, MODE_CHAN, MODE_INVALID = 0, 1, 2, 3, 4, 5, 0xFF
ST_POOL_FULL, ST_CORRUPT, ST_BAD_INDEX = 1, 2, 4

#: numpy view of kvc_desc
DESC_DTYPE = np.dtype([("off", "<u8"), ("scale", "<f4"), ("n16", "<u2"), ("mode", "u1"), ("rsvd", "u1")])

EXPORTS = ("kvc_create", "kvc_destroy", "kvc_set_scheme", "kvc_set_cache_layout", "kvc_bind_pool", "kvc_reset_pool", "kvc_restore_pool", "kvc_compress_blocks",
           "kvc_compress_blocks_mixed", "kvc_decompress_blocks", "kvc_gather_decompress", "kvc_set_prefetch_policy", "kvc_prefetch_reset", "kvc_prefetch_layers", "kvc_prefetch_window_workspace",
           "kvc_prefetch_layers_window", "kvc_prefetch_layers_window_static", "kvc_wall_clock_khz", "kvc_device_clocks", "kvc_stats", "kvc_page_scales",
           "kvc_copy_bytes", "kvc_strerror")


class Config(C.Structure):
    _fields_ = [("tokens_per_block", C.c_int32), ("head_dim", C.c_int32), ("pages_per_block", C.c_int32),
                ("scheme", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [("pool_bytes_used", C.c_uint64), ("pages", C.c_uint64 * 6), ("pages_invalid", C.c_uint64),
                ("payload_bytes", C.c_uint64), ("status", C.c_uint32), ("rsvd", C.c_uint32)]


class KvcError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {strerror(code)} ({code})")
        self.code = code


_lib = None


def load():
    """dlopen libkvc.so and declare the prototypes.  Raises if the library is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2512_11920_amd.build` "
                          "(there is no fallback implementation)")
    # libkvc.so needs the HIP runtime by soname; importing torch first makes the loader resolve it
    # to the copy torch already mapped, so tensors and kernels share one runtime instance.
    import torch  # noqa: F401

    L = C.CDLL(LIB_PATH)
    vp, i32p = C.c_void_p, C.c_void_p
    L.kvc_create.restype = C.c_int
    L.kvc_create.argtypes = [C.POINTER(vp), C.POINTER(Config)]
    L.kvc_destroy.restype = None
    L.kvc_destroy.argtypes = [vp]
    L.kvc_set_scheme.restype = C.c_int
    L.kvc_set_scheme.argtypes = [vp, C.c_int32]
    L.kvc_set_cache_layout.restype = C.c_int
    L.kvc_set_cache_layout.argtypes = [vp, C.c_int64, C.c_int64, C.c_int64]
    L.kvc_bind_pool.restype = C.c_int
    L.kvc_bind_pool.argtypes = [vp, vp, C.c_uint64, vp, C.c_uint64]
    L.kvc_reset_pool.restype = C.c_int
    L.kvc_reset_pool.argtypes = [vp, vp]
    L.kvc_restore_pool.restype = C.c_int
    L.kvc_restore_pool.argtypes = [vp, C.c_uint64, vp]
    L.kvc_compress_blocks.restype = C.c_int
    L.kvc_compress_blocks.argtypes = [vp, vp, C.c_int64, i32p, i32p, C.c_int32, vp]
    L.kvc_compress_blocks_mixed.restype = C.c_int
    L.kvc_compress_blocks_mixed.argtypes = [vp, vp, C.c_int64, i32p, i32p, vp, C.c_int32, vp]
    L.kvc_decompress_blocks.restype = C.c_int
    L.kvc_decompress_blocks.argtypes = [vp, vp, C.c_int64, i32p, i32p, C.c_int32, vp]
    L.kvc_gather_decompress.restype = C.c_int
    L.kvc_gather_decompress.argtypes = [vp, vp, i32p, C.c_int32, i32p, C.c_int32, C.c_int32, C.c_int32, C.c_int64, vp]
    L.kvc_set_prefetch_policy.restype = C.c_int
    L.kvc_set_prefetch_policy.argtypes = [vp, C.c_int32]
    L.kvc_prefetch_reset.restype = C.c_int
    L.kvc_prefetch_reset.argtypes = [vp, vp, C.c_int32, C.c_int32, C.c_int32, vp]
    L.kvc_prefetch_layers.restype = C.c_int
    L.kvc_prefetch_layers.argtypes = [vp, vp, vp, vp, vp, i32p, C.c_int32, i32p, i32p, C.c_int32, C.c_int32, C.c_int32,
                                      C.c_int32, C.c_int32, C.c_int64, C.c_int32, vp]
    L.kvc_prefetch_window_workspace.restype = C.c_uint64
    L.kvc_prefetch_window_workspace.argtypes = [C.c_int64, C.c_int32]
    L.kvc_prefetch_layers_window.restype = C.c_int
    L.kvc_prefetch_layers_window.argtypes = [vp, vp, vp, vp, vp, i32p, C.c_int32, i32p, i32p, C.c_int32, C.c_int32, C.c_int32,
                                             C.c_int32, C.c_int32, C.c_int64, C.c_int32, C.c_int32, vp, vp, C.c_uint64, vp]
    L.kvc_prefetch_layers_window_static.restype = C.c_int
    L.kvc_prefetch_layers_window_static.argtypes = [vp, vp, vp, vp, vp, i32p, C.c_int32, i32p, i32p, C.c_int32, C.c_int32, C.c_int32,
                                                    C.c_int32, C.c_int32, C.c_int64, C.c_int32, C.c_int32, vp, vp]
    L.kvc_wall_clock_khz.restype = C.c_int
    L.kvc_wall_clock_khz.argtypes = [C.POINTER(C.c_int32)]
    L.kvc_device_clocks.restype = C.c_int
    L.kvc_device_clocks.argtypes = [C.POINTER(C.c_int32)] * 3
    L.kvc_stats.restype = C.c_int
    L.kvc_stats.argtypes = [vp, C.POINTER(Stats), vp]
    L.kvc_page_scales.restype = C.c_int
    L.kvc_page_scales.argtypes = [vp, vp, vp, C.c_uint64, vp]
    L.kvc_copy_bytes.restype = C.c_int
    L.kvc_copy_bytes.argtypes = [vp, vp, C.c_uint64, vp]
    L.kvc_strerror.restype = C.c_char_p
    L.kvc_strerror.argtypes = [C.c_int]
    _lib = L
    return L


def strerror(code: int) -> str:
    return load().kvc_strerror(int(code)).decode()


def _check(rc: int, what: str):
    if rc != OK:
        raise KvcError(rc, what)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream(stream):
    import torch

    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def _ids(t):
    import torch

    if t is None:
        return None
    assert t.is_cuda and t.dtype == torch.int32 and t.is_contiguous(), "block ids: contiguous int32 CUDA tensor"
    return t


class Codec:
    """One kvc_ctx plus its bound pool and descriptor table (torch uint8 CUDA tensors)."""

    def __init__(self, tokens_per_block: int = 16, head_dim: int = 128, pages_per_block: int = 8, scheme: int = MODE_RLE):
        self._L = load()
        self.cfg = Config(tokens_per_block, head_dim, pages_per_block, scheme)
        self._ctx = C.c_void_p()
        _check(self._L.kvc_create(C.byref(self._ctx), C.byref(self.cfg)), "kvc_create")
        self.pool = None
        self.desc = None

    # -- geometry
    @property
    def page_elems(self) -> int:
        return self.cfg.tokens_per_block * self.cfg.head_dim

    @property
    def block_elems(self) -> int:
        return self.page_elems * self.cfg.pages_per_block

    def close(self):
        if self._ctx:
            self._L.kvc_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- pool
    def bind_pool(self, pool, desc):
        """pool: uint8 tensor, CUDA or pinned host memory (multiple of 16 bytes); desc: uint8 CUDA tensor of
        16*n_desc_pages bytes."""
        assert (pool.is_cuda or pool.is_pinned()) and desc.is_cuda and pool.is_contiguous() and desc.is_contiguous()
        assert pool.element_size() == 1 and desc.element_size() == 1 and desc.numel() % 16 == 0
        _check(self._L.kvc_bind_pool(self._ctx, pool.data_ptr(), pool.numel(), desc.data_ptr(), desc.numel() // 16),
               "kvc_bind_pool")
        self.pool, self.desc = pool, desc

    def alloc_pool(self, n_pool_blocks: int, pool_bytes: int, device="cuda:0", host_pool: bool = False):
        """host_pool: put the payload pool in pinned host memory (reached over the host link)."""
        import torch

        if host_pool:
            pool = torch.empty(int(pool_bytes) // 16 * 16, dtype=torch.uint8, pin_memory=True)
        else:
            pool = torch.empty(int(pool_bytes) // 16 * 16, dtype=torch.uint8, device=device)
        desc = torch.empty(int(n_pool_blocks) * self.cfg.pages_per_block * 16, dtype=torch.uint8, device=device)
        self.bind_pool(pool, desc)
        self.reset_pool()
        return pool, desc

    def reset_pool(self, stream=None):
        _check(self._L.kvc_reset_pool(self._ctx, _stream(stream)), "kvc_reset_pool")

    def restore_pool(self, used_bytes: int, stream=None):
        """Continue on a bound pool that holds an earlier run's payloads: the cursor resumes at used_bytes."""
        _check(self._L.kvc_restore_pool(self._ctx, int(used_bytes), _stream(stream)), "kvc_restore_pool")

    def set_scheme(self, scheme: int):
        _check(self._L.kvc_set_scheme(self._ctx, scheme), "kvc_set_scheme")
        self.cfg.scheme = scheme

    def set_cache_layout(self, block_stride: int = 0, page_stride: int = 0, row_stride: int = 0):
        """Strides (FP16 elements) of the cache buffers; all zero = contiguous [block][page][N][d]."""
        _check(self._L.kvc_set_cache_layout(self._ctx, block_stride, page_stride, row_stride), "kvc_set_cache_layout")
        self._block_stride = block_stride or self.block_elems
        self._span = ((self.cfg.pages_per_block - 1) * (page_stride or self.page_elems)
                      + (self.cfg.tokens_per_block - 1) * (row_stride or self.cfg.head_dim) + self.cfg.head_dim)

    # -- the three data calls
    def _blocks_of(self, t) -> int:
        """Number of whole blocks the tensor's storage covers under the current layout."""
        import torch

        assert t.is_cuda and t.is_contiguous() and t.dtype == torch.float16
        bs = getattr(self, "_block_stride", self.block_elems)
        span = getattr(self, "_span", self.block_elems)
        return 0 if t.numel() < span else (t.numel() - span) // bs + 1

    def compress_blocks(self, cache, n: int | None = None, src_ids=None, pool_ids=None, block_scheme=None, stream=None):
        """block_scheme: optional uint8 CUDA tensor, requested mode per block of the call."""
        import torch

        nb = self._blocks_of(cache)
        src_ids, pool_ids = _ids(src_ids), _ids(pool_ids)
        if n is None:
            n = src_ids.numel() if src_ids is not None else (pool_ids.numel() if pool_ids is not None else nb)
        assert all(t is None or t.numel() >= n for t in (src_ids, pool_ids)), "id tensors shorter than n"
        if block_scheme is None:
            _check(self._L.kvc_compress_blocks(self._ctx, cache.data_ptr(), nb, _ptr(src_ids), _ptr(pool_ids), int(n),
                                               _stream(stream)), "kvc_compress_blocks")
        else:
            assert block_scheme.is_cuda and block_scheme.dtype == torch.uint8 and block_scheme.numel() >= n
            _check(self._L.kvc_compress_blocks_mixed(self._ctx, cache.data_ptr(), nb, _ptr(src_ids), _ptr(pool_ids),
                                                     block_scheme.data_ptr(), int(n), _stream(stream)),
                   "kvc_compress_blocks_mixed")

    def decompress_blocks(self, out, n: int | None = None, pool_ids=None, dst_ids=None, stream=None):
        nb = self._blocks_of(out)
        pool_ids, dst_ids = _ids(pool_ids), _ids(dst_ids)
        if n is None:
            n = pool_ids.numel() if pool_ids is not None else (dst_ids.numel() if dst_ids is not None else nb)
        assert all(t is None or t.numel() >= n for t in (pool_ids, dst_ids)), "id tensors shorter than n"
        _check(self._L.kvc_decompress_blocks(self._ctx, out.data_ptr(), nb, _ptr(pool_ids), _ptr(dst_ids), int(n),
                                             _stream(stream)), "kvc_decompress_blocks")

    def gather_decompress(self, out, block_table, pred, n_layers: int, pool_blocks_per_layer: int, stream=None):
        block_table, pred = _ids(block_table), _ids(pred)
        n_seq, max_blocks = block_table.shape
        assert pred.shape[0] == n_seq
        k = pred.shape[1]
        assert self._blocks_of(out) == n_layers * n_seq * k
        _check(self._L.kvc_gather_decompress(self._ctx, out.data_ptr(), block_table.data_ptr(), max_blocks,
                                             pred.data_ptr(), n_seq, k, n_layers, int(pool_blocks_per_layer),
                                             _stream(stream)), "kvc_gather_decompress")

    def set_prefetch_policy(self, policy: int):
        """0: prediction j uses slot j; 1: wanted blocks stay put, missing ones take unwanted slots."""
        _check(self._L.kvc_set_prefetch_policy(self._ctx, policy), "kvc_set_prefetch_policy")

    def prefetch_reset(self, tags, n_seq: int, k: int, n_layers: int, stream=None):
        assert _ids(tags).numel() == 2 * n_layers * n_seq * k
        _check(self._L.kvc_prefetch_reset(self._ctx, tags.data_ptr(), n_seq, k, n_layers, _stream(stream)),
               "kvc_prefetch_reset")

    def prefetch_layers(self, l2, tags, fetch, loc, block_table, pred, n_layers: int, pool_blocks_per_layer: int,
                        fill_half: int, layer_begin: int = 0, layer_end: int | None = None, l1_first=None, stream=None):
        """l2: float16 [2][n_layers*n_seq*k][ppb][N][d]; tags int32 [2][n_slots]; fetch, loc int32 [n_slots]."""
        block_table, pred = _ids(block_table), _ids(pred)
        n_seq, max_blocks = block_table.shape
        k = pred.shape[1]
        n_slots = n_layers * n_seq * k
        assert self._blocks_of(l2) == 2 * n_slots
        assert _ids(tags).numel() == 2 * n_slots and _ids(fetch).numel() == n_slots and _ids(loc).numel() == n_slots
        assert pred.shape[0] == n_seq and (l1_first is None or l1_first.numel() == n_seq)
        layer_end = n_layers if layer_end is None else layer_end
        _check(self._L.kvc_prefetch_layers(self._ctx, l2.data_ptr(), tags.data_ptr(), fetch.data_ptr(), loc.data_ptr(),
                                           block_table.data_ptr(), max_blocks, pred.data_ptr(), _ptr(_ids(l1_first)),
                                           n_seq, k, n_layers, layer_begin, layer_end, int(pool_blocks_per_layer),
                                           fill_half, _stream(stream)), "kvc_prefetch_layers")

    def prefetch_layers_window(self, l2, tags, fetch, loc, block_table, pred, n_layers: int, pool_blocks_per_layer: int,
                               fill_half: int, omega: int, notify, work, layer_begin: int = 0, layer_end: int | None = None,
                               l1_first=None, stream=None):
        """prefetch_layers through the outstanding-request window: at most `omega` blocks in flight.
        notify: int64 CUDA tensor [n_layers + 4]; work: uint8 CUDA tensor of window_workspace(...) bytes, or
        None for the library's static workspace (kvc_prefetch_layers_window_static)."""
        import torch

        block_table, pred = _ids(block_table), _ids(pred)
        n_seq, max_blocks = block_table.shape
        k = pred.shape[1]
        n_slots = n_layers * n_seq * k
        assert self._blocks_of(l2) == 2 * n_slots
        assert _ids(tags).numel() == 2 * n_slots and _ids(fetch).numel() == n_slots and _ids(loc).numel() == n_slots
        assert pred.shape[0] == n_seq and (l1_first is None or l1_first.numel() == n_seq)
        assert notify.is_cuda and notify.dtype == torch.int64 and notify.numel() >= n_layers + 4 and notify.is_contiguous()
        assert work is None or (work.is_cuda and work.dtype == torch.uint8 and work.is_contiguous())
        layer_end = n_layers if layer_end is None else layer_end
        if work is None:  # the library's static workspace: the call that allocates nothing
            _check(self._L.kvc_prefetch_layers_window_static(
                self._ctx, l2.data_ptr(), tags.data_ptr(), fetch.data_ptr(), loc.data_ptr(), block_table.data_ptr(), max_blocks,
                pred.data_ptr(), _ptr(_ids(l1_first)), n_seq, k, n_layers, layer_begin, layer_end, int(pool_blocks_per_layer),
                fill_half, int(omega), notify.data_ptr(), _stream(stream)), "kvc_prefetch_layers_window_static")
            return
        _check(self._L.kvc_prefetch_layers_window(self._ctx, l2.data_ptr(), tags.data_ptr(), fetch.data_ptr(), loc.data_ptr(),
                                                  block_table.data_ptr(), max_blocks, pred.data_ptr(), _ptr(_ids(l1_first)),
                                                  n_seq, k, n_layers, layer_begin, layer_end, int(pool_blocks_per_layer),
                                                  fill_half, int(omega), notify.data_ptr(), work.data_ptr(), work.numel(),
                                                  _stream(stream)), "kvc_prefetch_layers_window")

    def stats(self, stream=None, check: bool = False) -> dict:
        st = Stats()
        rc = self._L.kvc_stats(self._ctx, C.byref(st), _stream(stream))
        if rc not in (OK, ERR_POOL_FULL, ERR_CORRUPT) or (check and rc != OK):
            raise KvcError(rc, "kvc_stats")
        return {"rc": rc, "pool_bytes_used": st.pool_bytes_used, "pages": list(st.pages),
                "pages_invalid": st.pages_invalid, "payload_bytes": st.payload_bytes, "status": st.status}

    # -- host views for tests and tools
    def desc_numpy(self) -> np.ndarray:
        return self.desc.cpu().numpy().view(DESC_DTYPE)

    def ratio(self) -> float:
        """R_c = uncompressed bytes / (payload + descriptor bytes) over stored pages (Section 3.5.2)."""
        s = self.stats()
        n = sum(s["pages"])
        return (n * self.page_elems * 2) / (s["payload_bytes"] + 16 * n) if n else float("nan")


def window_workspace(n_blocks: int, n_layers_call: int) -> int:
    """Bytes of device workspace prefetch_layers_window needs for a call over n_blocks slots."""
    return int(load().kvc_prefetch_window_workspace(int(n_blocks), int(n_layers_call)))


def device_clocks() -> dict:
    """Shader and memory clock (kHz) and memory bus width (bits) of the current device, as the runtime reports them."""
    a, b, c = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    _check(load().kvc_device_clocks(C.byref(a), C.byref(b), C.byref(c)), "kvc_device_clocks")
    return {"shader_khz": a.value, "memory_khz": b.value, "memory_bus_bits": c.value}


def wall_clock_khz() -> int:
    """Rate (kHz) of the device clock that the ready stamps of prefetch_layers_window count."""
    v = C.c_int32()
    _check(load().kvc_wall_clock_khz(C.byref(v)), "kvc_wall_clock_khz")
    return int(v.value)


def page_scales(amax_bits, stream=None):
    """Scaling step of Alg. 2 for FP16 page maxima (int16/uint16 CUDA tensor of bit patterns): -> (s, s_inv)."""
    import torch

    assert amax_bits.is_cuda and amax_bits.element_size() == 2 and amax_bits.is_contiguous()
    s = torch.empty(amax_bits.numel(), dtype=torch.float32, device=amax_bits.device)
    s_inv = torch.empty_like(s)
    _check(load().kvc_page_scales(amax_bits.data_ptr(), s.data_ptr(), s_inv.data_ptr(), amax_bits.numel(), _stream(stream)),
           "kvc_page_scales")
    return s, s_inv


def copy_bytes(dst, src, stream=None):
    """Yardstick copy kernel: dst[:] = src[:] (uint8 CUDA tensors, multiple of 16 bytes)."""
    assert dst.is_cuda and src.is_cuda and dst.is_contiguous() and src.is_contiguous()
    assert dst.numel() * dst.element_size() == src.numel() * src.element_size()
    _check(load().kvc_copy_bytes(dst.data_ptr(), src.data_ptr(), src.numel() * src.element_size(), _stream(stream)),
           "kvc_copy_bytes")
