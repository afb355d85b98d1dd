"""The resident-grid 3x3 kernels (one workgroup per compute unit walking over several output tiles) against the oracle.

The library picks them for large grids only, so the test forces them (`ss_debug_force_tile`) and caps the number of
workgroups (`ss_debug_limit_blocks`), which makes every workgroup of a small problem hand over from tile to tile:
with a cap of 1 a single workgroup computes the whole layer, with 3 the tiles are dealt out unevenly."""
import numpy as np
import pytest

from paper_2411_00288_amd import workloads as wl
from helpers import check_close, oracle_ref, run_gpu

pytestmark = pytest.mark.gpu

STREAM_TILES = [10, 11]          # 256 x 128 and 256 x 64 output tiles


def _L(N, H, W, cin, cout, s=1, p=1, dtype=wl.F16, act=wl.ACT_RELU, seed=0):
    return wl.Layer(f"n{N}h{H}w{W}c{cin}o{cout}s{s}d{dtype}a{act}", N=N, H=H, W=W, cin=cin, cout=cout, kh=3, kw=3,
                    stride=s, pad=p, dtype=dtype, korder=wl.K_CRS, act=act, mask="logits", seed=seed)


SHAPES = [
    _L(3, 14, 14, 64, 300),                                   # 2 chunks, two row tiles (the second ragged), 588 pixels
    _L(2, 15, 13, 96, 136, s=2, dtype=wl.BF16, seed=1),       # stride 2, 3 chunks, one ragged row tile, 56 pixels: a single ragged tile
    _L(2, 14, 14, 192, 256, act=wl.ACT_NONE, seed=3),         # 6 chunks, exactly one row tile
    _L(5, 9, 11, 32, 520, p=0, dtype=wl.BF16, act=wl.ACT_GELU, seed=4),   # a single chunk per tile, three row tiles, no padding
    _L(1, 40, 33, 64, 64, seed=5),                            # 1320 pixels: 11 tiles of 128 over few workgroups, a quarter-filled row tile
]


@pytest.mark.parametrize("cap", [None, 1, 3])
@pytest.mark.parametrize("tile", STREAM_TILES)
@pytest.mark.parametrize("L", SHAPES, ids=lambda L: L.name)
def test_stream_kernels_match_oracle(ss, force_tile, limit_blocks, L, tile, cap):
    d = wl.make_inputs(L)
    ref = oracle_ref(L, d)
    force_tile(tile)
    limit_blocks(cap)
    check_close(run_gpu(ss, L, d, sparse=True), ref, f"{L.name} sparse tile {tile} cap {cap}")
    check_close(run_gpu(ss, L, d, sparse=False), ref, f"{L.name} dense tile {tile} cap {cap}")


@pytest.mark.parametrize("cap", [None, 2])
@pytest.mark.parametrize("tile", STREAM_TILES)
def test_stream_kernels_are_bit_exact_on_integers(ss, force_tile, limit_blocks, tile, cap):
    L = _L(3, 10, 9, 64, 150, act=wl.ACT_NONE)
    assert L.K + 2 <= 2048
    d = wl.make_small_int_inputs(L, seed=tile)
    ref = oracle_ref(L, d)
    force_tile(tile)
    limit_blocks(cap)
    for sparse in (True, False):
        y = run_gpu(ss, L, d, sparse=sparse)
        assert np.array_equal(y.float().cpu().numpy().astype(np.float64), ref)


def test_stream_kernel_without_bias(ss, force_tile, limit_blocks):
    L = _L(2, 12, 12, 64, 128, seed=7)
    d = wl.make_inputs(L)
    d0 = dict(d, bias=np.zeros_like(d["bias"]))
    ref = oracle_ref(L, d0)
    force_tile(10)
    limit_blocks(2)
    check_close(run_gpu(ss, L, d, sparse=True, bias=False), ref, "no bias")
