"""Host logic of the row-kernel launch planning (lnpegn_plan_query touches no device): whatever the heuristics
choose, the plan must be one the kernels can run."""
import itertools

import pytest

from paper_2411_00999_amd import binding

SHAPES_B = (1, 2, 3, 8, 16, 31, 33, 64, 100, 128, 200, 255, 256, 257, 260, 300, 384, 511, 512, 513, 600, 700, 1000,
            1024, 4096)
SHAPES_T = (1, 2, 3, 4, 5, 7, 8, 9, 16, 17, 31, 32, 33, 48, 64, 100, 128, 130, 512, 2048, 4096)
SHAPES_D = (1, 8, 64, 256, 257, 576, 768, 960, 1001, 1024, 1280, 1536, 1600, 2048, 2560, 3072, 4096, 5120, 6144, 8192,
            9216, 12288, 16384, 20480)


def _check(B, T, D, dt, per_example, aligned, tuned=False):
    p = binding.plan_query(B, T, D, dt, per_example, aligned)
    E = 8 if dt == binding.BF16 else 4
    tag = (B, T, D, dt, per_example, aligned, p)
    rows = T if per_example else B * T
    assert p["rows_per_example"] == rows, tag
    C = p["chunks_per_example"]
    assert C >= 1 and p["chunks"] == (B * C if per_example else C), tag
    assert C <= max(1, rows // 4), tag                       # a chunk keeps four rows or more
    if p["vector_kernel"]:
        S, R, vpt = p["waves_per_row"], p["row_groups"], p["vectors_per_lane"]
        assert aligned and D % E == 0, tag
        assert 1 <= S <= 8 and R >= 1 and S * R <= 8, tag     # a workgroup has at most 512 threads ...
        if S <= 2 and vpt * E <= 8:
            assert S * R <= 4, tag                            # ... 256 for the instantiations built with that bound
        assert 1 <= vpt <= 32 // E and 64 * S * vpt * E >= D, tag
        assert 64 * S * (vpt - 1) * E < D or vpt == 1, tag    # no lane slot that is all padding
        assert rows < 2 * R or C <= max(1, rows // (2 * R)), tag   # every row group gets two rows or more
    else:
        assert not aligned or D % E != 0 or D // E > 64 * (32 // E) * 8, tag
    assert 0 < p["lds_bytes"] <= 160 * 1024, tag
    if p["rows_per_block"]:
        assert C > 1 and p["rows_per_block"] * C >= rows and p["rows_per_block"] * (C - 1) <= rows + C, tag
        assert tuned or p["stagger"] == 0, tag
    if not per_example:
        assert p["stagger"] == 0 and (tuned or p["rows_per_block"] == 0), tag
        assert p["row_kernel_emits_norms"] == 0 and p["examples_in_reduction"] == 0, tag
    else:
        assert tuned or 0 <= p["stagger"] < max(rows, 1) * 2, tag
        if p["row_kernel_emits_norms"]:
            assert C == 1 and p["examples_in_reduction"] == 0 and p["vector_kernel"], tag
        else:
            assert p["examples_in_reduction"] == B, tag
    assert 1 <= p["groups"] <= 16 and p["groups"] * p["chunks_per_group"] >= p["chunks"], tag
    assert (p["groups"] - 1) * p["chunks_per_group"] < p["chunks"], tag          # no empty group
    if p["chunks_per_xcd"]:
        assert p["chunks_per_xcd"] * 8 == p["chunks"], tag
    assert 0 < p["workspace_bytes"] <= binding.load().lnpegn_workspace_bytes(B, T, D, dt), tag
    assert p["workspace_bytes"] % 256 == 0, tag
    return p


@pytest.mark.parametrize("dt", [binding.BF16, binding.F32], ids=["bf16", "f32"])
def test_every_plan_is_runnable(dt):
    n = 0
    for B, T, D in itertools.product(SHAPES_B, SHAPES_T, SHAPES_D):
        if B * T * D > (1 << 33):
            continue
        for per_example, aligned in ((True, True), (False, True), (True, False), (False, False)):
            _check(B, T, D, dt, per_example, aligned)
            n += 1
    assert n > 10000


@pytest.mark.parametrize("tuning", [((0, 7),), ((0, 16384), (1, 16384)), ((1, 3),), ((2, 1),), ((2, 16),), ((2, 6), (5, 1)),
                                    ((5, 1),), ((5, 3),), ((8, 2),), ((8, 1), (3, 1000)), ((4, 2),), ((0, 513), (2, 8), (8, 2))])
def test_every_plan_is_runnable_under_the_tuning_overrides(tuning):
    keys = sorted({k for k, _ in tuning})
    try:
        for k, v in tuning:
            binding.set_tuning(k, v)
        for dt in (binding.BF16, binding.F32):
            for B, T, D in itertools.product((1, 3, 16, 33, 300, 512, 1000), (1, 5, 33, 64, 130, 2048),
                                             (8, 257, 768, 1024, 1600, 2048, 3072, 8192, 12288)):
                for per_example, aligned in ((True, True), (False, True), (True, False)):
                    _check(B, T, D, dt, per_example, aligned, tuned=True)
    finally:
        for k in keys:
            binding.set_tuning(k, 0)


def test_plans_of_the_benchmark_workloads():
    """The shapes the measurements are quoted on, pinned so that a change of heuristics shows up here."""
    q = binding.plan_query
    p = q(16, 2048, 2048, binding.BF16)
    assert (p["waves_per_row"], p["row_groups"], p["chunks"], p["rows_per_block"]) == (2, 3, 256, 0)
    assert q(16, 2048, 2048, binding.BF16, per_example=False)["chunks"] == 256
    p = q(512, 64, 1024, binding.BF16)
    assert (p["waves_per_row"], p["row_groups"], p["chunks"], p["row_kernel_emits_norms"]) == (1, 8, 512, 1)
    p = q(8, 4096, 8192, binding.BF16)
    assert (p["waves_per_row"], p["row_groups"], p["chunks"], p["chunks_per_xcd"]) == (8, 1, 512, 64)
    p = q(16, 2048, 2048, binding.F32)
    assert (p["waves_per_row"], p["row_groups"], p["vectors_per_lane"], p["chunks"]) == (2, 3, 4, 2048)
    p = q(300, 100, 1024, binding.BF16)                      # examples cut finer than one round of workgroups
    assert p["chunks_per_example"] == 5 and p["rows_per_block"] == 20
    # the other rules of the planning, one shape each (figures of the measurements they came from: the source)
    for shape, want in {
        (600, 64, 1024): (1, 4, 3, 22),      # a last round that would be a sixth full: three rounds of blocks instead
        (513, 64, 1024): (1, 4, 3, 22),
        (260, 128, 1024): (1, 4, 6, 22),     # half a round: three rounds
        (700, 48, 1024): (1, 8, 1, 0),       # a second round more than a third full: whole examples, eight rows at a time
        (1000, 32, 1024): (1, 8, 1, 0),
        (64, 512, 1024): (1, 4, 8, 64),      # more than 32 examples: blocks of rows
        (32, 1024, 2048): (2, 3, 8, 0),      # up to 32: every C-th row
        (16, 2048, 1280): (2, 4, 16, 0),     # two waves per row with lanes left over: four row groups
        (16, 2048, 3072): (3, 2, 16, 0),     # three waves per row: two row groups
        (16, 2048, 6144): (6, 1, 32, 0),     # six waves per row: two rounds
    }.items():
        p = q(*shape, binding.BF16)
        got = (p["waves_per_row"], p["row_groups"], p["chunks_per_example"], p["rows_per_block"])
        assert got == want, (shape, got, want)


def test_plan_follows_the_tuning_and_rejects_bad_arguments():
    import ctypes
    lib = binding.load()
    try:
        binding.set_tuning(0, 64)
        assert binding.plan_query(16, 2048, 2048, binding.BF16)["chunks"] == 64
        binding.set_tuning(8, 2)
        assert binding.plan_query(16, 2048, 2048, binding.BF16)["rows_per_block"] == 512
    finally:
        binding.set_tuning(0, 0)
        binding.set_tuning(8, 0)
    out = (ctypes.c_int64 * 16)()
    assert lib.lnpegn_plan_query(0, 1, 1, binding.BF16, 1, 1, out, 16) == 1
    assert lib.lnpegn_plan_query(1, 1, 1, 7, 1, 1, out, 16) == 2
    assert lib.lnpegn_plan_query(1, 1, 1, binding.BF16, 1, 1, None, 16) == 1
    out[3] = -5
    assert lib.lnpegn_plan_query(4, 128, 256, binding.F32, 1, 1, out, 3) == 0 and out[3] == -5   # only n_out values
