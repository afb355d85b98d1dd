"""Pins for the oracle's max pooling: a library routine (torch.nn.functional.max_pool2d on float64 NCHW copies),
a brute-force numpy evaluation with -inf borders, and closed forms."""
import numpy as np
import pytest
import torch

import oracle
from paper_2411_00288_amd import workloads as wl


@pytest.mark.parametrize("shape", [(2, 9, 7, 8, 3, 2, 1), (1, 8, 8, 16, 2, 2, 0), (3, 5, 6, 8, 3, 1, 1), (1, 7, 7, 8, 7, 1, 3)])
@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
def test_maxpool_matches_library_and_brute_force(shape, dtype):
    N, H, W, C, k, s, p = shape
    rng = np.random.default_rng(4)
    xb = wl.to_bits(rng.standard_normal((N, H, W, C), dtype=np.float32), dtype)
    y = oracle.maxpool2d(xb, dtype=dtype, k=k, stride=s, pad=p)
    xv = oracle.bits_to_double(xb, dtype)
    ref = torch.nn.functional.max_pool2d(torch.from_numpy(xv).permute(0, 3, 1, 2), k, s, p).permute(0, 2, 3, 1).numpy()
    assert np.array_equal(oracle.bits_to_double(y, dtype), ref)
    # brute force with -inf outside the image
    xp = np.full((N, H + 2 * p, W + 2 * p, C), -np.inf)
    xp[:, p:p + H, p:p + W] = xv
    Ho, Wo = (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1
    bf = np.empty((N, Ho, Wo, C))
    for ho in range(Ho):
        for wo in range(Wo):
            bf[:, ho, wo] = xp[:, ho * s:ho * s + k, wo * s:wo * s + k].reshape(N, -1, C).max(axis=1)
    assert np.array_equal(oracle.bits_to_double(y, dtype), bf)


def test_maxpool_closed_forms():
    # a single large value is seen by exactly the windows that cover it; all-negative inputs are not clipped by the border
    x = np.full((1, 6, 6, 8), -3.0, dtype=np.float32)
    x[0, 2, 3, 5] = 9.0
    y = oracle.bits_to_double(oracle.maxpool2d(wl.to_bits(x, wl.F16), k=3, stride=2, pad=1), wl.F16)
    assert y.shape == (1, 3, 3, 8)
    expect = np.full((1, 3, 3, 8), -3.0)
    expect[0, 1, 1:3, 5] = 9.0         # windows rows {1,2,3}, cols {1,2,3} and {3,4,5}
    assert np.array_equal(y, expect)
    # 1x1 window, stride 1: identity on the bits (NaN and -0 included)
    b = np.array([0x8000, 0x7E01, 0x3C00, 0xFC00, 0x0001, 0x8001, 0x7C00, 0x0000], dtype=np.uint16).reshape(1, 1, 1, 8)
    assert np.array_equal(oracle.maxpool2d(b, k=1, stride=1, pad=0), b)
