"""Pins for the oracle's direct convolution (Sec. 3.3 Eq. 4 / Eq. 6).

Each pin is something other than the oracle itself: the unfold+matmul reformulation (Eq. 5)
written separately in numpy, a float64 library convolution, closed forms (one-hot kernels,
all-ones), linearity, the 1x1 == matmul special case, and the exact values of the 16-bit formats.
"""
import itertools

import numpy as np
import pytest
import torch

import oracle
from paper_2411_00288_amd import workloads as wl


def _unfold_matmul(xf, Wmat_crs, cin, kh, kw, stride, pad):
    """Eq. (5): Y~ = W * U(X) with an explicit unfold, NHWC in/out, float64; W is [cout, K] CRS."""
    N, H, Wd, _ = xf.shape
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (Wd + 2 * pad - kw) // stride + 1
    xp = np.zeros((N, H + 2 * pad, Wd + 2 * pad, cin))
    xp[:, pad:pad + H, pad:pad + Wd, :] = xf
    cols = np.zeros((cin * kh * kw, N * Ho * Wo))
    for c, r, t in itertools.product(range(cin), range(kh), range(kw)):
        patch = xp[:, r:r + stride * (Ho - 1) + 1:stride, t:t + stride * (Wo - 1) + 1:stride, c]
        cols[(c * kh + r) * kw + t] = patch.reshape(-1)
    Y = Wmat_crs @ cols                       # [cout, L]
    return Y.T.reshape(N, Ho, Wo, -1)


def _crs_view(Wmat, cin, kh, kw, korder):
    """[cout, K] in `korder` -> [cout, K] in CRS order (pure re-indexing)."""
    cout = Wmat.shape[0]
    if korder == wl.K_CRS:
        return Wmat
    return Wmat.reshape(cout, kh, kw, cin).transpose(0, 3, 1, 2).reshape(cout, -1)


SHAPES = [  # N, H, W, cin, cout, k, stride, pad
    (1, 4, 4, 4, 3, 1, 1, 0),
    (2, 5, 4, 4, 5, 3, 1, 1),
    (1, 5, 5, 8, 2, 3, 2, 1),
    (2, 4, 5, 4, 4, 2, 2, 0),
    (1, 3, 3, 4, 1, 3, 1, 0),
    (1, 5, 3, 8, 3, 3, 2, 0),
    (1, 2, 2, 4, 2, 3, 1, 1),
]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("korder", [wl.K_CRS, wl.K_RSC])
@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
def test_eq4_equals_eq5_and_library_conv(shape, korder, dtype):
    N, H, Wd, cin, cout, k, s, p = shape
    L = wl.Layer("t", N=N, H=H, W=Wd, cin=cin, cout=cout, kh=k, kw=k, stride=s, pad=p, dtype=dtype,
                 korder=korder, mask="logits", seed=hash(shape) % 1000)
    d = wl.make_inputs(L)
    y = oracle.conv2d(d["x"], d["W"], d["M"], cin=cin, kh=k, kw=k, korder=korder, dtype=dtype,
                      bias=d["bias"], stride=(s, s), pad=(p, p), act=wl.ACT_NONE)
    xf = wl.from_bits(d["x"], dtype).astype(np.float64)
    Wm = wl.from_bits(d["W"], dtype).astype(np.float64) * d["M"]
    Wcrs = _crs_view(Wm, cin, k, k, korder)
    # (i)+(ii) Eq. 5/6: unfold + matmul with M (.) W
    y5 = _unfold_matmul(xf, Wcrs, cin, k, k, s, p) + d["bias"].astype(np.float64)
    np.testing.assert_allclose(y, y5, rtol=1e-12, atol=1e-12)
    # (vii) float64 library convolution on NCHW copies
    yt = torch.nn.functional.conv2d(torch.from_numpy(xf.transpose(0, 3, 1, 2).copy()),
                                    torch.from_numpy(Wcrs.reshape(cout, cin, k, k).copy()),
                                    torch.from_numpy(d["bias"].astype(np.float64)), stride=s, padding=p)
    np.testing.assert_allclose(y, yt.numpy().transpose(0, 2, 3, 1), rtol=1e-12, atol=1e-12)
    # ReLU is max(., 0)
    yr = oracle.conv2d(d["x"], d["W"], d["M"], cin=cin, kh=k, kw=k, korder=korder, dtype=dtype,
                       bias=d["bias"], stride=(s, s), pad=(p, p), act=wl.ACT_RELU)
    assert np.array_equal(yr, np.maximum(y, 0))
    # masked conv == dense conv of the already-masked matrix (Eq. 6)
    Wm_bits = np.where(d["M"] == 1, d["W"], 0).astype(np.uint16)
    yd = oracle.conv2d(d["x"], Wm_bits, None, cin=cin, kh=k, kw=k, korder=korder, dtype=dtype,
                       bias=d["bias"], stride=(s, s), pad=(p, p))
    assert np.array_equal(y, yd)
    # sampled-points entry agrees with the full tensor
    idx = np.random.default_rng(0).integers(0, y.size, size=min(50, y.size))
    yp = oracle.conv2d_points(d["x"], d["W"], d["M"], idx, cin=cin, kh=k, kw=k, korder=korder,
                              dtype=dtype, bias=d["bias"], stride=(s, s), pad=(p, p))
    np.testing.assert_allclose(yp, y.reshape(-1)[idx], rtol=1e-13, atol=1e-13)


def test_asymmetric_stride_and_pad_against_library():
    N, H, Wd, cin, cout, kh, kw = 2, 7, 6, 4, 3, 3, 1
    L = wl.Layer("t", N=N, H=H, W=Wd, cin=cin, cout=cout, kh=kh, kw=kw, mask="top2", seed=9)
    d = wl.make_inputs(L)
    y = oracle.conv2d(d["x"], d["W"], d["M"], cin=cin, kh=kh, kw=kw, stride=(2, 1), pad=(1, 0))
    xf = wl.from_bits(d["x"], 0).astype(np.float64)
    Wm = (wl.from_bits(d["W"], 0).astype(np.float64) * d["M"]).reshape(cout, cin, kh, kw)
    yt = torch.nn.functional.conv2d(torch.from_numpy(xf.transpose(0, 3, 1, 2).copy()), torch.from_numpy(Wm),
                                    stride=(2, 1), padding=(1, 0)).numpy().transpose(0, 2, 3, 1)
    np.testing.assert_allclose(y, yt, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("korder", [wl.K_CRS, wl.K_RSC])
def test_one_hot_kernel_is_a_shift_with_zero_border(korder):
    # W[o,c,r,t] = 1 for a single entry => y[..., o] = x shifted by (r - pad, t - pad) in channel c,
    # zero outside: pins cross-correlation (no flip), the padding rule and the flattening order.
    N, H, Wd, cin, cout, k, p = 1, 5, 6, 4, 2, 3, 1
    x = np.arange(N * H * Wd * cin, dtype=np.float32).reshape(N, H, Wd, cin) % 17 + 1
    xb = wl.to_bits(x, wl.F16)
    for (o, c, r, t) in [(0, 1, 0, 0), (1, 3, 2, 1), (0, 0, 1, 2), (1, 2, 2, 2)]:
        w = np.zeros((cout, cin, k, k), dtype=np.float32)
        w[o, c, r, t] = 1
        Wb = wl.flatten_weight(wl.to_bits(w, wl.F16), korder)
        y = oracle.conv2d(xb, Wb, None, cin=cin, kh=k, kw=k, korder=korder, pad=(p, p))
        exp = np.zeros((N, H, Wd, cout))
        for i, j in itertools.product(range(H), range(Wd)):
            ii, jj = i - p + r, j - p + t
            if 0 <= ii < H and 0 <= jj < Wd:
                exp[0, i, j, o] = x[0, ii, jj, c]
        assert np.array_equal(y, exp)


def test_one_hot_kernel_with_stride():
    N, H, Wd, cin, k, s, p = 1, 7, 7, 4, 3, 2, 1
    x = (np.arange(H * Wd * cin, dtype=np.float32).reshape(1, H, Wd, cin) % 13) + 1
    w = np.zeros((1, cin, k, k), dtype=np.float32)
    w[0, 2, 0, 2] = 1
    y = oracle.conv2d(wl.to_bits(x, 0), wl.flatten_weight(wl.to_bits(w, 0), 0), None, cin=cin, kh=k, kw=k,
                      stride=(s, s), pad=(p, p))
    assert y.shape == (1, 4, 4, 1)
    for ho, wo in itertools.product(range(4), range(4)):
        ii, jj = ho * s - p + 0, wo * s - p + 2
        exp = x[0, ii, jj, 2] if (0 <= ii < H and 0 <= jj < Wd) else 0
        assert y[0, ho, wo, 0] == exp


def test_all_ones_counts_taps_inside_the_image():
    # all-ones 3x3 kernel on all-ones input, pad 1: 9*cin interior, 6*cin edge, 4*cin corner
    cin, H = 4, 5
    xb = wl.to_bits(np.ones((1, H, H, cin), dtype=np.float32), wl.BF16)
    Wb = wl.to_bits(np.ones((1, cin * 9), dtype=np.float32), wl.BF16)
    y = oracle.conv2d(xb, Wb, None, cin=cin, kh=3, kw=3, dtype=wl.BF16, pad=(1, 1))[0, :, :, 0]
    assert y[2, 2] == 9 * cin and y[0, 2] == 6 * cin and y[2, 0] == 6 * cin
    assert y[0, 0] == y[0, -1] == y[-1, 0] == y[-1, -1] == 4 * cin
    # with a 2:4 mask exactly half of the taps survive in the interior
    M = np.tile(np.array([1, 0, 0, 1], dtype=np.uint8), (1, cin * 9 // 4))
    ym = oracle.conv2d(xb, Wb, M, cin=cin, kh=3, kw=3, dtype=wl.BF16, pad=(1, 1))[0, :, :, 0]
    assert ym[2, 2] == 9 * cin / 2


def test_pointwise_conv_is_a_matmul():
    L = wl.Layer("t", N=2, H=3, W=5, cin=32, cout=12, kh=1, kw=1, dtype=wl.BF16, mask="top2", seed=4)
    d = wl.make_inputs(L)
    y = oracle.conv2d(d["x"], d["W"], d["M"], cin=32, kh=1, kw=1, dtype=wl.BF16)
    X = wl.from_bits(d["x"], wl.BF16).astype(np.float64).reshape(-1, 32)
    Wm = wl.from_bits(d["W"], wl.BF16).astype(np.float64) * d["M"]
    np.testing.assert_allclose(y.reshape(-1, 12), X @ Wm.T, rtol=1e-12, atol=1e-13)
    # for 1x1 the two flattenings coincide
    y2 = oracle.conv2d(d["x"], d["W"], d["M"], cin=32, kh=1, kw=1, dtype=wl.BF16, korder=wl.K_RSC)
    assert np.array_equal(y, y2)


def test_linearity_in_x_and_w():
    # small integers: every operation is exact, so linearity holds bit for bit
    L = wl.Layer("t", N=1, H=5, W=5, cin=8, cout=4, kh=3, kw=3, pad=1)
    a = wl.make_small_int_inputs(L, seed=1)
    b = wl.make_small_int_inputs(L, seed=2)
    kw = dict(cin=8, kh=3, kw=3, pad=(1, 1))
    f = lambda xb, Wb: oracle.conv2d(xb, Wb, a["M"], **kw)
    xa, xb_ = wl.from_bits(a["x"], 0), wl.from_bits(b["x"], 0)
    assert np.array_equal(f(wl.to_bits(xa + xb_, 0), a["W"]), f(a["x"], a["W"]) + f(b["x"], a["W"]))
    wa, wb = wl.from_bits(a["W"], 0), wl.from_bits(b["W"], 0)
    assert np.array_equal(f(a["x"], wl.to_bits(wa + 2 * wb, 0)), f(a["x"], a["W"]) + 2 * f(a["x"], b["W"]))
    # scaling x by 2 doubles the output
    assert np.array_equal(f(wl.to_bits(2 * xa, 0), a["W"]), 2 * f(a["x"], a["W"]))


def test_dropped_weights_do_not_contribute():
    # changing W at masked-out positions changes nothing (the mask leaves W itself untouched)
    L = wl.Layer("t", N=1, H=4, W=4, cin=8, cout=4, kh=3, kw=3, pad=1, mask="logits", seed=3)
    d = wl.make_inputs(L)
    W2 = d["W"].copy()
    W2[d["M"] == 0] = 0x7BFF        # 65504, the largest finite fp16
    kw = dict(cin=8, kh=3, kw=3, pad=(1, 1), bias=d["bias"])
    assert np.array_equal(oracle.conv2d(d["x"], d["W"], d["M"], **kw), oracle.conv2d(d["x"], W2, d["M"], **kw))


def test_bias_and_relu_closed_form():
    xb = wl.to_bits(np.zeros((1, 2, 2, 4), dtype=np.float32), 0)
    Wb = wl.to_bits(np.ones((3, 4), dtype=np.float32), 0)
    bias = np.array([-1.5, 0.0, 2.25], dtype=np.float32)
    y = oracle.conv2d(xb, Wb, None, cin=4, kh=1, kw=1, bias=bias, act=wl.ACT_RELU)
    assert np.array_equal(y[0, 0, 0], [0.0, 0.0, 2.25])
    y = oracle.conv2d(xb, Wb, None, cin=4, kh=1, kw=1, bias=bias, act=wl.ACT_NONE)
    assert np.array_equal(y[0, 1, 1], [-1.5, 0.0, 2.25])


def test_sixteen_bit_formats_are_widened_exactly():
    # closed-form values of the two storage formats
    cases16 = {0x0000: 0.0, 0x3C00: 1.0, 0xC000: -2.0, 0x7BFF: 65504.0, 0x0400: 2.0 ** -14,
               0x0001: 2.0 ** -24, 0x03FF: 1023 * 2.0 ** -24, 0x3555: 0.333251953125, 0x7C00: np.inf}
    for bits, val in cases16.items():
        assert oracle.bits_to_double([bits], wl.F16)[0] == val
    assert np.isnan(oracle.bits_to_double([0x7E00], wl.F16)[0])
    assert np.signbit(oracle.bits_to_double([0x8000], wl.F16)[0])
    casesbf = {0x3F80: 1.0, 0xC000: -2.0, 0x0080: 2.0 ** -126, 0x0001: 2.0 ** -133, 0x7F7F: 3.3895313892515355e38,
               0x3EAB: 0.333984375}
    for bits, val in casesbf.items():
        assert oracle.bits_to_double([bits], wl.BF16)[0] == val
    # all 65536 fp16 patterns against numpy's float16
    allb = np.arange(65536, dtype=np.uint16)
    mine = oracle.bits_to_double(allb, wl.F16)
    ref = allb.view(np.float16).astype(np.float64)
    assert np.array_equal(mine, ref, equal_nan=True)


def test_output_shape_formula_and_empty_output():
    # same padding, odd kernel, stride 1 -> L = b*d output positions (Sec. 3.3)
    xb = np.zeros((1, 6, 9, 4), dtype=np.uint16)
    Wb = np.zeros((2, 4 * 25), dtype=np.uint16)
    assert oracle.conv2d(xb, Wb, None, cin=4, kh=5, kw=5, pad=(2, 2)).shape == (1, 6, 9, 2)
    assert oracle.conv2d(xb, Wb, None, cin=4, kh=5, kw=5, stride=(2, 2), pad=(0, 0)).shape == (1, 1, 3, 2)
    with pytest.raises(ValueError):
        oracle.conv2d(np.zeros((1, 2, 2, 4), dtype=np.uint16), Wb, None, cin=4, kh=5, kw=5)
