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
SOURCES = [os.path.join(CSRC, f) for f in ("lnpegn.hip", "lnpegn_rows_inst.hip", "linear_pegn.hip", "embedding_pegn.hip")]
HEADERS = [os.path.join(CSRC, h) for h in ("lnpegn_device.h", "lnpegn_rows.h", "lnpegn_finalize.h", "lnpegn_tracker.h",
                                           "lnpegn_launch.h")]
# translation units: (source, extra defines, object tag).  The row kernels are one source compiled four times.
UNITS = [("lnpegn.hip", [], "abi"),
         ("lnpegn_rows_inst.hip", ["-DLNPEGN_INST_BF16=1", "-DLNPEGN_INST_SAVED=0"], "rows_bf16_recompute"),
         ("lnpegn_rows_inst.hip", ["-DLNPEGN_INST_BF16=1", "-DLNPEGN_INST_SAVED=1"], "rows_bf16_saved"),
         ("lnpegn_rows_inst.hip", ["-DLNPEGN_INST_BF16=0", "-DLNPEGN_INST_SAVED=0"], "rows_f32_recompute"),
         ("lnpegn_rows_inst.hip", ["-DLNPEGN_INST_BF16=0", "-DLNPEGN_INST_SAVED=1"], "rows_f32_saved"),
         ("linear_pegn.hip", [], "linear"),
         ("embedding_pegn.hip", [], "embedding")]
HEADERS.append(os.path.join(os.path.dirname(HERE), "include", "lnpegn.h"))

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
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
    """Compile every HIP source (side by side, one hipcc each) and link liblnpegn.so; always recompiles."""
    import concurrent.futures as cf
    import shutil
    import tempfile
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmpdir = tempfile.mkdtemp(prefix="lnpegn_build_")
    try:
        def compile_one(unit):
            name, defines, tag = unit
            obj = os.path.join(tmpdir, tag + ".o")
            cmd = [hipcc, *HIPCC_FLAGS, *defines, *extra_flags, "-c", "-o", obj, os.path.join(CSRC, name)]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True)
            return obj
        with cf.ThreadPoolExecutor(max_workers=min(len(UNITS), os.cpu_count() or 4)) as ex:
            objs = list(ex.map(compile_one, UNITS))
        tmp = LIB + f".tmp{os.getpid()}"
        cmd = [hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", "-o", tmp, *objs]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        os.replace(tmp, LIB)
    finally:
        shutil.rmtree(tmpdir, ignore_errors=True)
    return LIB


def ensure_built() -> str:
    """Return the library path, building only if no library exists yet."""
    if not os.path.exists(LIB):
        build()
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra_flags=sys.argv[1:])
    print(LIB)
