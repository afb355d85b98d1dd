"""Pins for the oracle's depthwise convolution: a float64 library grouped convolution, the dense oracle convolution
with a diagonal weight (Eq. 4 restricted to its diagonal), and a one-hot closed form."""
import numpy as np
import pytest
import torch

import oracle
from paper_2411_00288_amd import workloads as wl


@pytest.mark.parametrize("shape", [(2, 9, 8, 8, 7, 7, 3), (1, 6, 7, 16, 3, 3, 1), (2, 5, 5, 8, 5, 3, 0), (1, 8, 6, 8, 3, 5, 2)])
@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
def test_dwconv_matches_library_grouped_conv_and_diagonal_dense_conv(shape, dtype):
    N, H, W, C, kh, kw, p = shape
    rng = np.random.default_rng(9)
    xb = wl.to_bits(rng.standard_normal((N, H, W, C), dtype=np.float32), dtype)
    wb = wl.to_bits(rng.standard_normal((kh, kw, C), dtype=np.float32), dtype)
    bias = rng.standard_normal(C).astype(np.float32)
    y = oracle.dwconv2d(xb, wb, dtype=dtype, bias=bias, pad=(p, p), act=wl.ACT_RELU)
    xv, wv = oracle.bits_to_double(xb, dtype), oracle.bits_to_double(wb, dtype)
    ref = torch.nn.functional.conv2d(torch.from_numpy(xv).permute(0, 3, 1, 2), torch.from_numpy(wv).permute(2, 0, 1)[:, None],
                                     torch.from_numpy(bias.astype(np.float64)), padding=p, groups=C)
    ref = torch.relu(ref).permute(0, 2, 3, 1).numpy()
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)
    # the same numbers from the dense oracle convolution with a diagonal [C][C*kh*kw] weight
    Wd = np.zeros((C, C, kh, kw), dtype=np.uint16)
    for c in range(C):
        Wd[c, c] = wb[:, :, c]
    yd = oracle.conv2d(xb, Wd.reshape(C, -1), None, cin=C, kh=kh, kw=kw, dtype=dtype, bias=bias, pad=(p, p), act=wl.ACT_RELU)
    assert np.allclose(y, yd, rtol=1e-12, atol=1e-12)


def test_dwconv_one_hot_filter_is_a_per_channel_shift():
    x = np.arange(2 * 5 * 6 * 8, dtype=np.float32).reshape(2, 5, 6, 8) % 13
    w = np.zeros((3, 3, 8), dtype=np.float32)
    w[0, 2, 3] = 1.0        # channel 3 looks up-right; every other channel sees nothing
    y = oracle.dwconv2d(wl.to_bits(x, wl.F16), wl.to_bits(w, wl.F16), pad=(1, 1))
    expect = np.zeros_like(y)
    expect[:, 1:, :-1, 3] = x[:, :-1, 1:, 3]
    assert np.array_equal(y, expect)
