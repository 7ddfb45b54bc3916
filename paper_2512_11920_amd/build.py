"""Build libkvc.so (HIP, gfx950) in-tree with hipcc.  No GPU is needed to compile.

The codec kernels (csrc/kvc_codec.hip) are compiled once per group of page shapes
(-DKVC_SHAPE_GROUP=k), side by side with the other sources; the objects are then linked."""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
_CSRC = os.path.join(_PKG, "csrc")
SHAPE_GROUPS = 16  # see csrc/kvc_codec.hip
#: (source, extra defines, object name)
UNITS = [("kvc_kernels.hip", (), "kvc_kernels.o"), ("kvc_api.hip", (), "kvc_api.o")] + \
        [("kvc_codec.hip", (f"-DKVC_SHAPE_GROUP={g}",), f"kvc_codec_{g}.o") for g in range(SHAPE_GROUPS)]
SOURCES = [os.path.join(_CSRC, f) for f in ("kvc_kernels.hip", "kvc_codec.hip", "kvc_api.hip")]
HEADERS = [os.path.join(_CSRC, f) for f in ("kvc_common.h", "kvc_device.h", "kvc_codec.h")] + [os.path.join(_ROOT, "include", "kvc.h")]
LIB = os.path.join(_PKG, "libkvc.so")
#: the same library with every LDS index and pool span the kernels compute checked against its bounds
#: (a violation sets status bit 8); a GPU test runs the parity cases through it
LIB_DEBUG = os.path.join(_PKG, "libkvc_dbg.so")
OBJ_DIR = os.path.join(_PKG, "_build")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # no packed-FP32 code generation
    "-Wall", "-Wno-unused-command-line-argument",
]
INCLUDES = ["-I", os.path.join(_ROOT, "include"), "-I", _CSRC]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def _hipcc() -> str:
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def compile_unit(source: str, defines=(), out: str | None = None, extra_flags=(), asm: bool = False, verbose: bool = False) -> str:
    """Compile one source of csrc/ to an object (or, with asm=True, to the gfx950 assembly of its kernels)."""
    mode = ["-S", "--cuda-device-only"] if asm else ["-c"]
    cmd = [_hipcc(), *HIPCC_FLAGS, *extra_flags, *defines, *INCLUDES, *mode, "-o", out, os.path.join(_CSRC, source)]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {source} {' '.join(defines)}:\n{err}")
    if err.strip():
        print(err, file=sys.stderr)
    return out


def build(force: bool = True, verbose: bool = False, extra_flags=(), lib: str = LIB, jobs: int | None = None) -> str:
    if not force and not stale():
        return lib
    obj_dir = OBJ_DIR if lib == LIB else os.path.join(OBJ_DIR, os.path.basename(lib) + ".objs")
    os.makedirs(obj_dir, exist_ok=True)
    jobs = jobs or max(1, min(len(UNITS), os.cpu_count() or 1, 16))
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        futs = [ex.submit(compile_unit, src, defs, os.path.join(obj_dir, obj), tuple(extra_flags), False, verbose)
                for src, defs, obj in UNITS]
        objs = [f.result() for f in futs]
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-Wno-unused-command-line-argument", "-o", lib, *objs]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    subprocess.run(cmd, check=True)
    return lib


def build_debug(verbose: bool = False) -> str:
    return build(force=True, verbose=verbose, extra_flags=("-DKVC_DEBUG_BOUNDS=1",), lib=LIB_DEBUG)


CLIENT_SRC = os.path.join(_ROOT, "tests", "abi_client.cpp")
CLIENT_BIN = os.path.join(_ROOT, "tests", "abi_client")


def build_client(verbose: bool = False) -> str:
    """Compile the stand-alone C-ABI client (HIP runtime + kvc.h only) against the built library."""
    cmd = [_hipcc(), "-O2", "-std=c++17", "-Wall", "-Wno-unused-command-line-argument", "-I", os.path.join(_ROOT, "include"),
           "-o", CLIENT_BIN, CLIENT_SRC, "-L", _PKG, "-lkvc", "-Wl,-rpath," + _PKG, "-Wl,-rpath,$ORIGIN/../paper_2512_11920_amd"]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    subprocess.run(cmd, check=True)
    return CLIENT_BIN


if __name__ == "__main__":
    print(build(force=True, verbose=True))
    print(build_debug(verbose=True))
    print(build_client(verbose=True))
