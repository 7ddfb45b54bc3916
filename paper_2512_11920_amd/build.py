"""Build libkvc.so (HIP, gfx950) in-tree with hipcc.  No GPU is needed to compile."""
from __future__ import annotations

import os
import subprocess
import sys

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
SOURCES = [os.path.join(_PKG, "csrc", f) for f in ("kvc_kernels.hip", "kvc_page16.hip", "kvc_api.hip")]
HEADERS = [os.path.join(_PKG, "csrc", "kvc_common.h"), os.path.join(_PKG, "csrc", "kvc_device.h"),
           os.path.join(_ROOT, "include", "kvc.h")]
LIB = os.path.join(_PKG, "libkvc.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # no packed-FP32 code generation
    "-Wall", "-Wno-unused-command-line-argument",
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False, extra_flags=()) -> str:
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(_ROOT, "include"), "-I", os.path.join(_PKG, "csrc"),
           "-o", LIB, *SOURCES]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    subprocess.run(cmd, check=True)
    return LIB


CLIENT_SRC = os.path.join(_ROOT, "tests", "abi_client.cpp")
CLIENT_BIN = os.path.join(_ROOT, "tests", "abi_client")


def build_client(verbose: bool = False) -> str:
    """Compile the stand-alone C-ABI client (HIP runtime + kvc.h only) against the built library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O2", "-std=c++17", "-Wall", "-Wno-unused-command-line-argument", "-I", os.path.join(_ROOT, "include"),
           "-o", CLIENT_BIN, CLIENT_SRC, "-L", _PKG, "-lkvc", "-Wl,-rpath," + _PKG, "-Wl,-rpath,$ORIGIN/../paper_2512_11920_amd"]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    subprocess.run(cmd, check=True)
    return CLIENT_BIN


if __name__ == "__main__":
    print(build(force=True, verbose=True))
    print(build_client(verbose=True))
