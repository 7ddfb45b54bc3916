"""MI355X-native KV-cache page codec (compression / decompression engine of CXL-SpecKV).

``kvc``   ctypes binding of the HIP library (libkvc.so); no fallback path.
``synth`` seeded synthetic KV caches and access patterns.
``build`` compiles the library in-tree with hipcc for gfx950.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "kvc", "build"]
