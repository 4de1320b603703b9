"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the header
declares, sizes workspaces, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2411_00999_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "lnpegn.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return re.findall(r"^(?:int|size_t|const char \*)\s*\*?(\w+)\s*\(", text, flags=re.M)


def test_header_functions_are_exported():
    names = _declared_functions()
    assert set(names) == set(binding.EXPORTS), names
    lib = binding.load()
    for name in names:
        assert getattr(lib, name) is not None


def test_workspace_bytes_is_a_pure_host_function():
    lib = binding.load()
    for B, T, D, dt in ((4, 128, 256, 0), (8, 1024, 768, 1), (16, 2048, 2048, 1), (512, 64, 1024, 1),
                        (8, 4096, 8192, 1), (1, 1, 1, 0), (3, 5, 1001, 1)):
        n = lib.lnpegn_workspace_bytes(B, T, D, dt)
        assert n > 0 and n % 256 == 0
        assert n >= 2 * D * 4            # at least one chunk vector
    assert lib.lnpegn_workspace_bytes(0, 1, 1, 0) == 0
    assert lib.lnpegn_workspace_bytes(1, -1, 1, 0) == 0
    assert lib.lnpegn_workspace_bytes(1, 1, 0, 1) == 0
    assert lib.lnpegn_workspace_bytes(1, 1, 1, 7) == 0
    # the workspace of the headline workload stays a small fraction of the streamed bytes
    assert lib.lnpegn_workspace_bytes(16, 2048, 2048, 1) < 0.1 * 3 * 16 * 2048 * 2048 * 2


def test_workspace_stays_a_fraction_of_the_streamed_bytes():
    """A chunk ends with a write of 2*D fp32 column sums, so a chunk must keep a few rows: whatever the launch
    heuristics choose, the workspace of a launch that streams 32 MiB or more in examples of 64 rows or more stays
    below 0.4 of the bytes streamed (the worst cases are a handful of very wide rows per chunk)."""
    lib = binding.load()
    for dt, esz in ((binding.BF16, 2), (binding.F32, 4)):
        for B in (1, 2, 3, 8, 16, 33, 64, 100, 128, 200, 260, 300, 384, 512, 513, 600, 1000, 4096):
            for T in (64, 100, 128, 512, 2048):
                for D in (64, 256, 768, 1024, 1600, 2048, 4096, 8192, 12288, 1001):
                    streamed = 3 * B * T * D * esz
                    if streamed >= (32 << 20):
                        ws = lib.lnpegn_workspace_bytes(B, T, D, dt)
                        assert 0 < ws <= 0.4 * streamed, (B, T, D, dt, ws, streamed)


def test_status_strings():
    lib = binding.load()
    seen = {lib.lnpegn_status_string(i) for i in range(5)}
    assert len(seen) == 5 and all(s for s in seen)
    assert lib.lnpegn_status_string(99) == b"unknown status"


def test_bad_arguments_are_rejected_before_any_launch():
    """Every call below fails validation on the host, so no kernel is launched and the fake
    pointers are never dereferenced."""
    lib = binding.load()
    P = ctypes.c_void_p
    fake = [P(0x1000 * (i + 1)) for i in range(12)]
    x, dy, g, mean, rstd, dx, dg, db, sg, sb, big, ws = fake
    ws = P(0x100000)
    big_ws = 1 << 40

    def bwd(**kw):
        a = dict(x=x, dy=dy, g=g, mean=None, rstd=None, dx=dx, dg=dg, db=db, B=2, T=3, D=8, dt=1,
                 gdt=1, eps=1e-5, ws=ws, wsb=big_ws)
        a.update(kw)
        return lib.ln_bwd(a["x"], a["dy"], a["g"], a["mean"], a["rstd"], a["dx"], a["dg"], a["db"],
                          a["B"], a["T"], a["D"], a["dt"], a["gdt"], a["eps"], a["ws"], a["wsb"], None)

    EINVAL, EUNSUP, EWS = 1, 2, 3
    assert bwd(B=0) == EINVAL
    assert bwd(T=-4) == EINVAL
    assert bwd(D=0) == EINVAL
    assert bwd(eps=-1.0) == EINVAL
    assert bwd(eps=float("nan")) == EINVAL
    assert bwd(x=None) == EINVAL
    assert bwd(dy=None) == EINVAL
    assert bwd(g=None) == EINVAL
    assert bwd(dx=None) == EINVAL
    assert bwd(dg=None) == EINVAL
    assert bwd(db=None) == EINVAL
    assert bwd(dx=x) == EINVAL                       # dx must not alias x
    assert bwd(mean=mean) == EINVAL                  # mean and rstd come together
    assert bwd(dt=5) == EUNSUP
    assert bwd(gdt=-1) == EUNSUP
    assert bwd(ws=None) == EWS
    assert bwd(wsb=16) == EWS
    assert bwd(ws=P(0x100010)) == EINVAL             # workspace not 256-byte aligned

    def pegn(**kw):
        a = dict(sg=sg, sb=sb, B=2)
        a.update(kw)
        return lib.ln_bwd_pegn(x, dy, g, None, None, dx, dg, db, a["sg"], a["sb"], big, a["B"], 3, 8, 1,
                               1, 1e-5, ws, big_ws, None)

    assert pegn(sg=None) == EINVAL
    assert pegn(sb=None) == EINVAL
    assert pegn(B=0) == EINVAL

    assert lib.ln_fwd_stats(None, mean, rstd, 2, 3, 8, 1, 1e-5, None) == EINVAL
    assert lib.ln_fwd_stats(x, None, rstd, 2, 3, 8, 1, 1e-5, None) == EINVAL
    assert lib.ln_fwd_stats(x, mean, rstd, 2, 0, 8, 1, 1e-5, None) == EINVAL
    assert lib.ln_fwd_stats(x, mean, rstd, 2, 3, 8, 9, 1e-5, None) == EUNSUP

    out = fake[3]
    assert lib.gns_estimate(None, big, 1, 4, 4.0, out, None) == EINVAL
    assert lib.gns_estimate(sg, None, 1, 4, 4.0, out, None) == EINVAL
    assert lib.gns_estimate(sg, big, 1, 4, 4.0, None, None) == EINVAL
    assert lib.gns_estimate(sg, big, 0, 4, 4.0, out, None) == EINVAL
    assert lib.gns_estimate(sg, big, 1, 1, 1.0, out, None) == EINVAL   # B_big == B_small

    assert lib.lnpegn_set_tuning(99, 1) == EINVAL
    assert lib.lnpegn_set_tuning(0, -1) == EINVAL
    assert lib.lnpegn_set_tuning(0, 1 << 30) == EINVAL
    assert lib.lnpegn_set_tuning(2, 17) == EINVAL
    assert lib.lnpegn_set_tuning(7, 3) == EINVAL
    assert lib.lnpegn_set_tuning(8, 3) == EINVAL
    assert lib.lnpegn_set_tuning(8, 2) == 0 and lib.lnpegn_set_tuning(8, 0) == 0
    assert lib.lnpegn_set_tuning(0, 0) == 0


def test_tuning_changes_workspace_query():
    lib = binding.load()
    base = lib.lnpegn_workspace_bytes(16, 2048, 2048, 1)
    try:
        assert lib.lnpegn_set_tuning(0, 256) == 0
        assert lib.lnpegn_set_tuning(1, 256) == 0
        assert lib.lnpegn_workspace_bytes(16, 2048, 2048, 1) < base
    finally:
        lib.lnpegn_set_tuning(0, 0)
        lib.lnpegn_set_tuning(1, 0)
    assert lib.lnpegn_workspace_bytes(16, 2048, 2048, 1) == base


def test_workloads_are_seeded_and_representable():
    import numpy as np
    from paper_2411_00999_amd import workloads
    a = workloads.make_inputs(2, B=2, T=8, D=768)
    b = workloads.make_inputs(2, B=2, T=8, D=768)
    assert np.array_equal(a.x, b.x) and np.array_equal(a.dy, b.dy)
    workloads.bf16_bits(a.x), workloads.bf16_bits(a.dy), workloads.bf16_bits(a.gamma)   # raise if not
    c = workloads.make_inputs(3, layer=1, B=2, T=8, D=64)
    d = workloads.make_inputs(3, layer=2, B=2, T=8, D=64)
    assert not np.array_equal(c.x, d.x)
    e = workloads.make_inputs(4, B=8, T=4, D=32)
    assert np.array_equal(e.x[0], e.x[3]) and not np.array_equal(e.x[0], e.x[4])
    f = workloads.make_inputs(5, B=1, T=64, D=800)
    col_rms = np.sqrt((f.x[0].astype(np.float64) ** 2).mean(0))
    assert int((col_rms > 10).sum()) == 8              # 1% of the channels carry the x20 outliers
    r = workloads.round_to_bf16(np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0078125], np.float32))
    assert np.array_equal(r, np.array([1.0, 1.015625, 1.0078125], np.float32))  # ties to even


def test_linear_accum_steps_host_function_matches_oracle():
    """Host-only integer arithmetic: callable without a GPU."""
    import numpy as np
    from oracle import gns_tracker_oracle as trk
    from paper_2411_00999_amd import binding
    rng = np.random.default_rng(3)
    cases = [(0, 800, 8), (1, 800, 8), (101, 800, 8), (799, 800, 8), (800, 800, 8), (5, 0, 7), (0, 0, 1),
             (2 ** 62, 2 ** 63 - 1, 2 ** 31 - 1)]
    cases += [(int(t), int(r), int(a)) for t, r, a in zip(rng.integers(0, 2 ** 62, 300),
                                                          rng.integers(1, 2 ** 62, 300), rng.integers(1, 2 ** 20, 300))]
    for t, r, a in cases:
        assert binding.gns_linear_accum_steps(t, r, a) == trk.linear_accum_steps(t, r, a), (t, r, a)
    import pytest
    for bad in [(-1, 10, 2), (1, -10, 2), (1, 10, 0)]:
        with pytest.raises(binding.LnpegnError):
            binding.gns_linear_accum_steps(*bad)


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU only: any other --gpus ends with a message and a non-zero status, before
    anything touches a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr or "one GPU" in r.stderr


def test_product_path_does_not_import_the_oracle():
    """The oracle is test infrastructure: nothing under the package may import it."""
    pkg = os.path.join(ROOT, "paper_2411_00999_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            text = open(os.path.join(pkg, name)).read()
            assert "import oracle" not in text and "from oracle" not in text, name
    for name in os.listdir(os.path.join(pkg, "csrc")):
        text = open(os.path.join(pkg, "csrc", name)).read()
        assert "oracle/" not in text, name


def test_header_compiles_alone_as_c():
    """The public header is self-contained C: a translation unit that includes nothing else."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    for std in ("c99", "c11"):
        r = subprocess.run([gcc, f"-std={std}", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c",
                            HEADER], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


def test_c_program_calls_the_library(tmp_path):
    """tests/c_caller/abi_caller.c, built with gcc against the header and liblnpegn.so, runs the host-only
    entry points and the argument-validation paths from plain C."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    binding.load()
    lib = binding.lib_path()
    exe = str(tmp_path / "abi_caller")
    src = os.path.join(ROOT, "tests", "c_caller", "abi_caller.c")
    libdir = os.path.dirname(lib)
    r = subprocess.run([gcc, "-std=c11", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"), src,
                        "-o", exe, "-L", libdir, "-l:liblnpegn.so", f"-Wl,-rpath,{libdir}",
                        "-Wl,-rpath-link,/opt/rocm/lib"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "all checks passed" in r.stdout
