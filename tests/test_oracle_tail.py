"""Pins for the oracle's layer tail: residual add before the activation, ReLU and exact GELU.

None of these re-types the oracle's formula: they use closed forms with zero weights, an identity of the
GELU, tabulated values of the standard normal CDF, and a library CDF (scipy).
"""
import numpy as np
import pytest
from scipy.stats import norm

import oracle
from paper_2411_00288_amd import workloads as wl

pytestmark = pytest.mark.filterwarnings("ignore::RuntimeWarning")


def _zero_weight_layer(z, dtype=wl.F16, act=wl.ACT_NONE):
    """Runs z (values exactly representable in `dtype`, shape [N,H,W,C]) through a layer whose weights are all
    zero, so that the pre-activation equals the residual: returns act(residual)."""
    N, H, W, C = z.shape
    xb = wl.to_bits(np.ones((N, H, W, 4), dtype=np.float32), dtype)
    Wb = wl.to_bits(np.zeros((C, 4), dtype=np.float32), dtype)
    return oracle.conv2d(xb, Wb, None, cin=4, kh=1, kw=1, dtype=dtype, residual=wl.to_bits(z, dtype), act=act)


def test_residual_is_added_before_the_activation():
    rng = np.random.default_rng(5)
    z = rng.integers(-8, 9, size=(2, 3, 3, 5)).astype(np.float32)            # exact in fp16
    assert np.array_equal(_zero_weight_layer(z), z)                          # identity: plain copy of the residual
    assert np.array_equal(_zero_weight_layer(z, act=wl.ACT_RELU), np.maximum(z, 0))
    # bias -3 on a residual of +2: ReLU sees -1 (0 out); applied the other way round it would give 2
    xb = wl.to_bits(np.zeros((1, 1, 1, 4), dtype=np.float32), wl.F16)
    Wb = wl.to_bits(np.zeros((2, 4), dtype=np.float32), wl.F16)
    res = wl.to_bits(np.array([[[[2.0, 5.0]]]], dtype=np.float32), wl.F16)
    y = oracle.conv2d(xb, Wb, None, cin=4, kh=1, kw=1, bias=np.array([-3.0, -3.0], dtype=np.float32), residual=res,
                      act=wl.ACT_RELU)
    assert np.array_equal(y[0, 0, 0], [0.0, 2.0])


def test_residual_layout_is_nhwc_of_the_output():
    # one-hot residual at (n, ho, wo, o): it must come out at exactly that output element (stride-2 conv so the
    # output shape differs from the input's)
    N, H, W, C, cout = 2, 5, 7, 4, 3
    xb = wl.to_bits(np.zeros((N, H, W, C), dtype=np.float32), wl.F16)
    Wb = wl.to_bits(np.zeros((cout, C * 9), dtype=np.float32), wl.F16)
    Ho, Wo = 3, 4
    for (n, ho, wo, o) in [(0, 0, 0, 0), (1, 2, 3, 2), (0, 1, 2, 1), (1, 0, 3, 0)]:
        r = np.zeros((N, Ho, Wo, cout), dtype=np.float32)
        r[n, ho, wo, o] = 7.0
        y = oracle.conv2d(xb, Wb, None, cin=C, kh=3, kw=3, stride=(2, 2), pad=(1, 1), residual=wl.to_bits(r, wl.F16))
        assert y.shape == (N, Ho, Wo, cout) and np.array_equal(y, r)
        idx = np.array([((n * Ho + ho) * Wo + wo) * cout + o, 0 if (n, ho, wo, o) != (0, 0, 0, 0) else 5])
        pts = oracle.conv2d_points(xb, Wb, None, idx, cin=C, kh=3, kw=3, stride=(2, 2), pad=(1, 1),
                                   residual=wl.to_bits(r, wl.F16))
        assert np.array_equal(pts, [7.0, 0.0])


def test_residual_adds_to_a_real_convolution():
    L = wl.Layer("t", N=2, H=6, W=5, cin=8, cout=12, kh=3, kw=3, stride=1, pad=1, dtype=wl.BF16, korder=wl.K_CRS,
                 act=wl.ACT_NONE, mask="logits", seed=11)
    inp = wl.make_inputs(L)
    rng = np.random.default_rng(3)
    r = rng.integers(-4, 5, size=(2, 6, 5, 12)).astype(np.float32)
    kw = dict(cin=8, kh=3, kw=3, dtype=wl.BF16, bias=inp["bias"], stride=(1, 1), pad=(1, 1))
    plain = oracle.conv2d(inp["x"], inp["W"], inp["M"], **kw)
    fused = oracle.conv2d(inp["x"], inp["W"], inp["M"], residual=wl.to_bits(r, wl.BF16), **kw)
    assert np.allclose(fused - plain, r, rtol=0, atol=1e-12)
    fused_relu = oracle.conv2d(inp["x"], inp["W"], inp["M"], residual=wl.to_bits(r, wl.BF16), act=wl.ACT_RELU, **kw)
    assert np.array_equal(fused_relu, np.maximum(fused, 0))
    idx = np.arange(0, fused.size, 7)
    pts = oracle.conv2d_points(inp["x"], inp["W"], inp["M"], idx, residual=wl.to_bits(r, wl.BF16), act=wl.ACT_RELU, **kw)
    assert np.array_equal(pts, fused_relu.reshape(-1)[idx])


def test_gelu_identity_table_and_library_cdf():
    z = np.array([0.0, 0.5, 1.0, 2.0, 3.0, 0.25, 6.0, -0.5, -1.0, -2.0, -3.0, -0.25, -6.0, 1.5, -1.5, 4.0],
                 dtype=np.float32).reshape(1, 4, 4, 1)                      # all exact in fp16
    g = _zero_weight_layer(z, act=wl.ACT_GELU).reshape(-1)
    zz = z.reshape(-1).astype(np.float64)
    lut = dict(zip(zz, g))
    # gelu(z) - gelu(-z) = z * (Phi(z) + Phi(-z)) = z
    for v in (0.5, 1.0, 2.0, 3.0, 0.25, 6.0, 1.5):
        assert abs((lut[v] - lut[-v]) - v) < 1e-15 * max(1.0, v)
    assert lut[0.0] == 0.0
    # tabulated standard normal CDF: Phi(1) = 0.8413447461, Phi(2) = 0.9772498681, Phi(3) = 0.9986501020
    assert abs(lut[1.0] - 0.8413447461) < 1e-9
    assert abs(lut[2.0] - 2 * 0.9772498681) < 1e-9
    assert abs(lut[3.0] - 3 * 0.9986501020) < 1e-9
    assert abs(lut[-1.0] + (1 - 0.8413447461)) < 1e-9
    # far tails: identity / zero
    assert abs(lut[6.0] - 6.0) < 1e-8 and abs(lut[-6.0]) < 1e-8
    # library CDF on everything
    assert np.allclose(g, zz * norm.cdf(zz), rtol=1e-13, atol=1e-15)


def test_gelu_after_bias_and_residual_on_a_convolution():
    L = wl.Layer("t", N=1, H=4, W=4, cin=16, cout=8, kh=1, kw=1, stride=1, pad=0, dtype=wl.F16, korder=wl.K_CRS,
                 act=wl.ACT_NONE, mask="top2", seed=2)
    inp = wl.make_inputs(L)
    r = wl.to_bits(np.full((1, 4, 4, 8), 0.5, dtype=np.float32), wl.F16)
    kw = dict(cin=16, kh=1, kw=1, dtype=wl.F16, bias=inp["bias"])
    pre = oracle.conv2d(inp["x"], inp["W"], inp["M"], residual=r, **kw)
    g = oracle.conv2d(inp["x"], inp["W"], inp["M"], residual=r, act=wl.ACT_GELU, **kw)
    assert np.allclose(g, pre * norm.cdf(pre), rtol=1e-13, atol=1e-15)
