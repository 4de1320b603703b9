"""Build the lnpegn shared library for gfx950 with hipcc (cross-compiles without a GPU).

    python -m paper_2411_00999_amd.build          # rebuild liblnpegn.so in-tree
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblnpegn.so")
SOURCES = [os.path.join(CSRC, f) for f in ("lnpegn.hip", "linear_pegn.hip", "embedding_pegn.hip")]
HEADERS = [os.path.join(CSRC, h) for h in ("lnpegn_device.h", "lnpegn_rows.h", "lnpegn_finalize.h", "lnpegn_tracker.h")]
HEADERS.append(os.path.join(os.path.dirname(HERE), "include", "lnpegn.h"))

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # no packed-fp32 instructions: plain scalar fp32 code generation only
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every HIP source into liblnpegn.so (always recompiles)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-o", tmp, *SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    return LIB


def ensure_built() -> str:
    """Return the library path, building only if no library exists yet."""
    if not os.path.exists(LIB):
        build()
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra_flags=sys.argv[1:])
    print(LIB)
