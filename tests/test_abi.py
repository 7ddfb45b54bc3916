"""The C-ABI library loads here (no GPU), exports every symbol include/kvc.h declares, and its
host-side argument checks answer before any device work."""
import ctypes as C
import os
import re

import pytest

from paper_2512_11920_amd import kvc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "kvc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvc_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_three_hot_path_calls():
    names = _declared()
    for n in ("kvc_compress_blocks", "kvc_decompress_blocks", "kvc_gather_decompress"):
        assert n in names


def test_library_exports_every_declared_symbol():
    lib = kvc.load()
    names = _declared()
    assert len(names) >= 11
    for n in names:
        assert hasattr(lib, n), f"libkvc.so does not export {n}"
    assert sorted(kvc.EXPORTS) == names, "binding and header disagree on the entry points"


def test_descriptor_and_config_layouts():
    assert kvc.DESC_DTYPE.itemsize == 16
    assert [kvc.DESC_DTYPE.fields[f][1] for f in ("off", "scale", "n16", "mode", "rsvd")] == [0, 8, 12, 14, 15]
    assert C.sizeof(kvc.Config) == 16 and C.sizeof(kvc.Stats) == 80


def test_host_side_argument_checks_need_no_device():
    lib = kvc.load()
    ctx = C.c_void_p()
    assert lib.kvc_create(None, None) == kvc.ERR_ARG
    assert lib.kvc_create(C.byref(ctx), None) == kvc.ERR_ARG
    for cfg, want in ((kvc.Config(0, 128, 1, 3), kvc.ERR_ARG), (kvc.Config(16, 128, 0, 3), kvc.ERR_ARG),
                      (kvc.Config(16, 128, 1, -1), kvc.ERR_ARG), (kvc.Config(16, 100, 1, 3), kvc.ERR_ARG),
                      (kvc.Config(16, 288, 1, 3), kvc.ERR_UNSUPPORTED), (kvc.Config(64, 128, 1, 3), kvc.ERR_UNSUPPORTED),
                      (kvc.Config(16, 96, 1, 5), kvc.ERR_UNSUPPORTED),
                      (kvc.Config(16, 160, 1, 5), kvc.ERR_UNSUPPORTED), (kvc.Config(8, 128, 1, 5), kvc.ERR_UNSUPPORTED),
                      (kvc.Config(8, 256, 1, 5), kvc.ERR_UNSUPPORTED),
                      (kvc.Config(16, 128, 1, 6), kvc.ERR_ARG)):
        assert lib.kvc_create(C.byref(ctx), C.byref(cfg)) == want
        assert not ctx.value
    assert lib.kvc_set_scheme(None, 1) == kvc.ERR_ARG
    assert lib.kvc_set_cache_layout(None, 0, 0, 0) == kvc.ERR_ARG
    assert lib.kvc_bind_pool(None, None, 0, None, 0) == kvc.ERR_ARG
    assert lib.kvc_reset_pool(None, None) == kvc.ERR_ARG
    assert lib.kvc_restore_pool(None, 0, None) == kvc.ERR_ARG
    assert lib.kvc_compress_blocks(None, None, 0, None, None, 0, None) == kvc.ERR_ARG
    assert lib.kvc_compress_blocks_mixed(None, None, 0, None, None, None, 0, None) == kvc.ERR_ARG
    assert lib.kvc_decompress_blocks(None, None, 0, None, None, 0, None) == kvc.ERR_ARG
    assert lib.kvc_gather_decompress(None, None, None, 0, None, 0, 0, 0, 0, None) == kvc.ERR_ARG
    assert lib.kvc_set_prefetch_policy(None, 0) == kvc.ERR_ARG
    assert lib.kvc_prefetch_reset(None, None, 0, 0, 0, None) == kvc.ERR_ARG
    assert lib.kvc_prefetch_layers(None, None, None, None, None, None, 0, None, None, 0, 0, 0, 0, 0, 0, 0, None) == kvc.ERR_ARG
    assert lib.kvc_stats(None, None, None) == kvc.ERR_ARG
    assert lib.kvc_page_scales(None, None, None, 4, None) == kvc.ERR_ARG
    assert lib.kvc_page_scales(None, None, None, 0, None) == 0  # nothing to do
    assert lib.kvc_copy_bytes(None, None, 16, None) == kvc.ERR_ARG
    assert lib.kvc_copy_bytes(C.c_void_p(4096), C.c_void_p(8192), 24, None) == kvc.ERR_ARG  # not a multiple of 16
    lib.kvc_destroy(None)


def test_strerror_covers_every_code():
    seen = set()
    for code in range(0, -7, -1):
        msg = kvc.strerror(code)
        assert msg and msg != "unknown error"
        seen.add(msg)
    assert len(seen) == 7
    assert kvc.strerror(-99) == "unknown error"


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(kvc, "_lib", None)
    monkeypatch.setattr(kvc, "LIB_PATH", str(tmp_path / "libkvc.so"))
    with pytest.raises(ImportError):
        kvc.load()
