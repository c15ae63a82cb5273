"""The workgroup-id -> tile mapping of the token loss's matrix-core kernels, checked exhaustively on the
CPU: the mapping header is pure integer code, compiled here with g++ into a small harness.  For every
grid shape the kernels can be launched with, every tile must be taken by exactly one workgroup id (two
would race on d_hidden, none would leave a tile of the result unwritten)."""
import ctypes
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def harness(tmp_path_factory):
    out = tmp_path_factory.mktemp("tile_map") / "libtile_map_check.so"
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Werror",
                           "-I", os.path.join(ROOT, "paper_2504_13818_amd", "csrc"),
                           os.path.join(ROOT, "tests", "tile_map_check.cpp"), "-o", str(out)])
    lib = ctypes.CDLL(str(out))
    i64 = ctypes.c_int64
    lib.tile_map_check_one.argtypes = [i64, i64]
    lib.tile_map_check_ids.argtypes = [i64, i64, i64]
    lib.tile_map_check_range.argtypes = [i64, i64, i64, i64, ctypes.POINTER(i64)]
    lib.tile_map_check_range.restype = i64
    lib.strip_map_check_one.argtypes = [i64, i64]
    lib.strip_map_check_range.argtypes = [i64, i64, i64, i64, ctypes.POINTER(i64)]
    lib.strip_map_check_range.restype = i64
    lib.strip_map_used.argtypes = [i64]
    for name in ("tile_map_blocks", "tile_map_grid"):
        getattr(lib, name).argtypes = [i64, i64]
        getattr(lib, name).restype = i64
    lib.tile_map_few_blocks.restype = i64
    return lib


def _sweep(lib, lo, hi, step, n1_hi):
    first = (ctypes.c_int64 * 3)(0, 0, 0)
    bad = lib.tile_map_check_range(lo, hi, step, n1_hi, first)
    assert bad == 0, f"{bad} grids fail; first: n0={first[0]} n1={first[1]} code={first[2]}"


def test_every_grid_up_to_the_token_tiles_of_the_benchmark_shapes(harness):
    """Token tiles (n0) up to 2100 x second axis up to 40: covers the forward launches (up to 32
    vocabulary tiles per launch at the default chunk) and d_hidden (up to 16 d-tiles at d = 4096), on
    both sides of the few-blocks switch."""
    _sweep(harness, 1, 2100, 1, 40)     # includes 576, 1152, 2048: the capacities R*T/256 of the benchmark shapes


def test_wide_second_axis(harness):
    """Up to 130 tiles on the second axis: vocabulary chunks of up to 32768 columns, d up to 16384 and beyond."""
    _sweep(harness, 1, 140, 1, 130)
    _sweep(harness, 141, 2100, 61, 130)


def test_both_branches_are_exercised(harness):
    few = harness.tile_map_few_blocks()
    assert harness.tile_map_blocks(16, 8) < few <= harness.tile_map_blocks(1152, 8)
    assert harness.tile_map_blocks(252, 8) < few == harness.tile_map_blocks(253, 8)
    # the launches of the Qwen2.5-3B-shaped benchmark: 1152 token-tile capacity x 32 vocabulary tiles / 8 d-tiles
    for n0, n1 in ((1152, 32), (1152, 18), (1152, 8), (32, 8), (36, 14), (32, 16), (2048, 14), (1024, 16)):
        assert harness.tile_map_check_one(n0, n1) == 0
        assert harness.tile_map_grid(n0, n1) >= n0 * n1


def test_the_check_sees_a_broken_launch(harness):
    """The checker itself: a launch one XCD round short of the mapping's own size leaves tiles unnamed, in
    both branches; a full launch is accepted."""
    for n0, n1 in ((4, 8), (1152, 8)):
        grid = harness.tile_map_grid(n0, n1)
        assert harness.tile_map_check_ids(n0, n1, grid) == 0
        assert harness.tile_map_check_ids(n0, n1, grid - 8) == 3
        assert harness.tile_map_check_ids(n0, n1, grid - 3) == 4


def test_strip_mapping_of_d_w_lm(harness):
    """d_w_lm with many vocabulary tiles (n0) launches one round of 256 workgroup ids at a time under its own
    mapping: every tile exactly once, and the 32 workgroups an XCD gets in a round stay within 16 operand
    columns.  Vocabulary tiles up to 1100 (V = 281 600) x d-tiles up to 64 (d = 16384)."""
    first = (ctypes.c_int64 * 3)(0, 0, 0)
    bad = harness.strip_map_check_range(1, 1100, 1, 64, first)
    assert bad == 0, f"{bad} grids fail; first: n0={first[0]} n1={first[1]} code={first[2]}"
    # the benchmark heads (594 and 501 vocabulary tiles) take this mapping, small vocabularies the general one
    assert harness.strip_map_used(594) == 1 and harness.strip_map_used(501) == 1 and harness.strip_map_used(40) == 0
    for n0, n1 in ((594, 8), (594, 14), (501, 16)):
        assert harness.strip_map_check_one(n0, n1) == 0
