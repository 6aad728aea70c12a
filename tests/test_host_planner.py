"""CPU-side checks of the host logic that shapes the projection launches (no GPU needed): the plan must
cover every row and the whole contraction for any shape, keep the kernel's structural assumptions, and pick
the measured-best shapes at the two benchmark models."""
import itertools
import os

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2509_23094_amd", "libd2c.so")
pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="libd2c.so not built (run __graft_entry__.build())")


def _plan(*a, **k):
    from paper_2509_23094_amd import binding as B
    return B.d2c_plan_projection(*a, **k)


ROWS = [1, 15, 16, 17, 46, 64, 69, 96, 127, 128, 129, 150, 160, 161, 185, 192, 193, 200, 256, 257, 300, 512, 640,
        856, 1024, 3072, 12288]
SHAPES = [(12288, 4096), (4096, 4096), (24576, 4096), (4096, 12288), (126464, 4096),          # LLaDA-8B
          (4608, 3584), (3584, 3584), (37888, 3584), (3584, 18944), (152064, 3584),           # Dream-7B
          (768, 256), (1376, 256), (256, 688), (40, 20), (100, 132), (200, 264), (3000, 520), (33000, 256), (144, 64)]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_plan_covers_rows_and_contraction_and_keeps_the_kernel_assumptions(dtype):
    elem_per_chunk = 128 if dtype == "bf16" else 64
    for (N, K), m, single in itertools.product(SHAPES, ROWS, (False, True)):
        if K % (8 if dtype == "bf16" else 4):
            continue                                   # the launcher refuses rows that are not whole 16-byte pieces
        p = _plan(dtype, m, N, K, single)
        where = f"{dtype} m={m} N={N} K={K} single={single}: {p}"
        assert p["row_tiles"] * 16 * p["row_chunks"] >= m, where
        assert (p["row_tiles"] * 16) * (p["row_chunks"] - 1) < m, where              # no empty row chunk
        assert p["k_per_split"] * p["splits"] >= K and p["k_per_split"] * (p["splits"] - 1) < K, where
        assert p["k_per_split"] % elem_per_chunk == 0, where                        # splits start on chunk boundaries
        assert 1 <= p["splits"] <= 8 and (not single or p["splits"] == 1), where
        assert p["waves"] in (4, 6, 7, 8, 10) and p["col_tiles_per_wave"] in (1, 2, 4), where
        cols = 16 * p["col_tiles_per_wave"] * p["waves"]
        assert p["workgroups"] == -(-N // cols) * p["splits"] * p["row_chunks"], where
        if p["col_tiles_per_wave"] == 4:
            # the hand-pipelined loop for many rows: bf16, 6-8 row tiles per chunk, 4 waves, chunks taken in pairs
            assert dtype == "bf16" and p["row_tiles"] in (6, 7, 8) and p["waves"] == 4 and m >= 257, where
            assert K % 256 == 0 and p["k_per_split"] % 256 == 0, where
            # fewer than 8 tiles only with as many row chunks as 8 tiles need, or with whole blocks of 8 chunks
            tiles = -(-m // 16)
            assert p["row_tiles"] == 8 or p["row_chunks"] == -(-tiles // 8) or p["row_chunks"] % 8 == 0, where
        if p["row_tiles"] > 8:
            # the tall single chunk: bf16 only, even tile counts up to 12, 8 waves, one column tile per wave
            assert dtype == "bf16" and p["row_tiles"] in (10, 12) and p["row_chunks"] == 1, where
            assert p["waves"] == 8 and p["col_tiles_per_wave"] == 1 and 129 <= m <= 192, where
        if p["row_chunks"] == 1 and p["row_tiles"] <= 8:
            assert p["row_tiles"] == -(-m // 16), where


def test_plan_rows_per_workgroup_for_many_rows():
    """The measured cases of the rows-per-workgroup rule (LLaDA widths)."""
    for m, tiles, chunks in ((288, 6, 3), (400, 7, 4), (512, 8, 4), (700, 6, 8), (856, 7, 8), (1000, 8, 8),
                             (1100, 8, 9), (1500, 6, 16), (2048, 8, 16), (12288, 8, 96)):
        for (N, K) in ((12288, 4096), (4096, 12288)):
            p = _plan("bf16", m, N, K)
            assert (p["row_tiles"], p["row_chunks"]) == (tiles, chunks), (m, N, K, p)


def test_plan_at_the_benchmark_shapes():
    """One round of equal workgroups over the 256 compute units where the shape allows it (the shapes
    measured fastest on the MI355X)."""
    # LLaDA-8B, 46 rows
    assert _plan("bf16", 46, 12288, 4096)["workgroups"] == 256 and _plan("bf16", 46, 12288, 4096)["waves"] == 6
    assert _plan("bf16", 46, 4096, 4096)["workgroups"] == 256 and _plan("bf16", 46, 4096, 4096)["splits"] == 8
    gu = _plan("bf16", 46, 24576, 4096, True)
    assert (gu["workgroups"], gu["waves"], gu["splits"]) == (256, 6, 1)
    assert _plan("bf16", 46, 4096, 12288)["workgroups"] == 256
    # Dream-7B, 69 rows: the gate/up projection in one round of 10-wave workgroups instead of 296 8-wave ones
    gu = _plan("bf16", 69, 37888, 3584, True)
    assert (gu["workgroups"], gu["waves"], gu["splits"]) == (237, 10, 1)
    assert _plan("bf16", 69, 4608, 3584)["workgroups"] == 252
    # 3584 output columns: 7-wave workgroups (112 columns) make 32 column blocks x 8 splits = one full round
    dn = _plan("bf16", 69, 3584, 18944)
    assert (dn["waves"], dn["splits"], dn["workgroups"]) == (7, 8, 256)
    assert _plan("bf16", 69, 37888, 3584, True)["waves"] != 7        # the gated epilogue pairs neighbouring waves
    # row-count regimes
    assert _plan("bf16", 150, 12288, 4096)["row_tiles"] == 10 and _plan("bf16", 185, 12288, 4096)["row_tiles"] == 12
    p = _plan("bf16", 200, 12288, 4096)
    assert (p["row_chunks"], p["col_tiles_per_wave"]) == (2, 2)
    p = _plan("bf16", 856, 12288, 4096)
    assert (p["row_tiles"], p["row_chunks"], p["col_tiles_per_wave"], p["waves"]) == (7, 8, 4, 4)
    p = _plan("f32", 856, 768, 256)
    assert p["col_tiles_per_wave"] == 2 and p["row_chunks"] == 7


def test_plan_rejects_bad_arguments():
    from paper_2509_23094_amd import binding as B
    import ctypes
    shape = (ctypes.c_int32 * 7)()
    assert B._lib.d2c_plan_projection(1, 0, 16, 16, 0, shape) == B.D2C_EINVAL
    assert B._lib.d2c_plan_projection(5, 4, 16, 16, 0, shape) == B.D2C_EINVAL
    assert B._lib.d2c_plan_projection(1, 4, 16, 16, 0, None) == B.D2C_EINVAL
