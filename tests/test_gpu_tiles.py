"""Every instantiated tile shape / prefetch depth of the convolution kernel against the oracle.

The library picks a tile from the problem size; the test hook `ss_debug_force_tile(id)` (include/ss_debug.h)
forces one, so each shape is exercised here on problems that span several tiles in both
directions and leave ragged tails, for every staging mode, sparse and dense.
"""

import numpy as np
import pytest
import torch

from paper_2411_00288_amd import workloads as wl
from helpers import check_close, oracle_ref, run_gpu

pytestmark = pytest.mark.gpu

TILE_IDS = [0, 1, 2, 3, 4, 5]


def _L(N, H, W, cin, cout, k, s=1, p=0, dtype=wl.F16, korder=wl.K_CRS, seed=0):
    return wl.Layer(f"n{N}h{H}w{W}c{cin}o{cout}k{k}s{s}d{dtype}o{korder}", N=N, H=H, W=W, cin=cin, cout=cout, kh=k, kw=k,
                    stride=s, pad=p, dtype=dtype, korder=korder, act=wl.ACT_RELU, mask="logits", seed=seed)


SHAPES = [
    _L(3, 14, 14, 64, 300, 3, p=1),                        # tap transpose, 3 chunks of 32 channels... (2), ragged rows and pixels
    _L(2, 15, 13, 96, 136, 3, s=2, p=1, dtype=wl.BF16),    # stride 2, 3 chunks, bf16
    _L(3, 9, 11, 160, 264, 1, dtype=wl.BF16),              # pointwise, K = 160 (ragged 128-chunk), ragged everything
    _L(2, 10, 10, 64, 130, 1),                             # pointwise, short reduction (2 steps)
    _L(2, 12, 12, 96, 200, 2, s=2),                        # 2x2 stride 2 tap transpose
    _L(2, 9, 9, 24, 140, 3, p=1, korder=wl.K_RSC),         # channels-last flattening with taps
    _L(2, 9, 9, 64, 140, 3, p=1, korder=wl.K_RSC, seed=5), # channels-last flattening, K = 576: chunks of 256 (2.25 of them)
    _L(1, 11, 9, 12, 150, 3, p=1),                         # gather fallback (cin % 32 != 0)
    _L(2, 19, 17, 4, 70, 7, s=2, p=3, korder=wl.K_RSC, seed=9),   # 4-channel image, 7x7 stride 2: one 8-byte load per block, K = 196
    _L(1, 9, 10, 20, 150, 3, p=1, korder=wl.K_RSC, seed=8),       # cin % 8 == 4 in the channels-last flattening
    _L(2, 14, 14, 192, 260, 3, p=1, seed=3),               # six chunks of 32 channels
]


@pytest.mark.parametrize("tile", TILE_IDS)
@pytest.mark.parametrize("L", SHAPES, ids=lambda L: L.name)
def test_every_tile_shape_matches_oracle(ss, force_tile, L, tile):
    d = wl.make_inputs(L)
    ref = oracle_ref(L, d)
    force_tile(tile)
    check_close(run_gpu(ss, L, d, sparse=True), ref, f"{L.name} sparse tile {tile}")
    check_close(run_gpu(ss, L, d, sparse=False), ref, f"{L.name} dense tile {tile}")


@pytest.mark.parametrize("tile", TILE_IDS)
def test_every_tile_shape_is_bit_exact_on_integers(ss, force_tile, tile):
    L = _L(3, 10, 9, 64, 150, 3, p=1)
    L = wl.Layer(**{**L.__dict__, "act": wl.ACT_NONE})
    assert L.K + 2 <= 2048
    d = wl.make_small_int_inputs(L, seed=tile)
    ref = oracle_ref(L, d)
    force_tile(tile)
    for sparse in (True, False):
        y = run_gpu(ss, L, d, sparse=sparse)
        assert np.array_equal(y.float().cpu().numpy().astype(np.float64), ref)
