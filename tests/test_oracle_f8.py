"""Pins of the oracle's FP8 (OCP E4M3) functions (CPU only)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2411_00288_amd import workloads as wl


def _layer(**kw):
    base = dict(name="t", N=2, H=6, W=5, cin=8, cout=6, kh=3, kw=3, stride=1, pad=1, dtype=wl.F8, korder=wl.K_RSC,
                mask="logits", seed=3)
    base.update(kw)
    return wl.Layer(**base)


def test_every_byte_decodes_like_the_library_format():
    b = np.arange(256, dtype=np.uint8)
    got = oracle.e4m3_to_double(b)
    lib = torch.from_numpy(b.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(got), np.isnan(lib)) and np.isnan(got).sum() == 2
    ok = ~np.isnan(got)
    assert np.array_equal(got[ok], lib[ok]) and np.array_equal(np.signbit(got[ok]), np.signbit(lib[ok]))
    # closed forms of the format: 1.0, the largest value, the smallest subnormal and normal, -0, monotone magnitudes
    assert got[0x38] == 1.0 and got[0x7E] == 448.0 and got[0x01] == 2.0 ** -9 and got[0x08] == 2.0 ** -6
    assert got[0x80] == 0.0 and np.signbit(got[0x80]) and got[0xFE] == -448.0
    assert (np.diff(got[:0x7F]) > 0).all()
    assert np.array_equal(got[0x80:0xFF], -got[0x00:0x7F])


@pytest.mark.parametrize("korder", [wl.K_CRS, wl.K_RSC])
@pytest.mark.parametrize("geom", [dict(), dict(stride=2, pad=0), dict(kh=1, kw=1, pad=0, cin=12), dict(kh=2, kw=2, stride=2, pad=0)])
def test_agrees_with_the_binary16_oracle_on_the_same_values(korder, geom):
    """Every E4M3 value is exact in binary16, and both functions sum exact products in fp64 in the same loop order."""
    L = _layer(korder=korder, act=wl.ACT_RELU, **geom)
    d = wl.make_inputs_f8(L)
    x16 = wl.to_bits(oracle.e4m3_to_double(d["x"]).astype(np.float32), wl.F16)
    W16 = wl.to_bits(oracle.e4m3_to_double(d["W"]).astype(np.float32), wl.F16)
    assert np.array_equal(wl.from_bits(x16, wl.F16).astype(np.float64), oracle.e4m3_to_double(d["x"]))
    kw = dict(cin=L.cin, kh=L.kh, kw=L.kw, korder=korder, bias=d["bias"], stride=(L.stride,) * 2, pad=(L.pad,) * 2,
              act=wl.ACT_RELU)
    ref = oracle.conv2d(x16, W16, d["M"], dtype=wl.F16, **kw)
    got = oracle.conv2d_f8(d["x"], d["W"], d["M"], **kw)
    assert np.array_equal(got, ref)
    got_dense = oracle.conv2d_f8(d["x"], d["W"], None, **kw)
    assert np.array_equal(got_dense, oracle.conv2d(x16, W16, None, dtype=wl.F16, **kw))


def test_scale_bias_activation_and_points():
    L = _layer(N=2, H=7, W=7, cin=8, cout=10, stride=2)
    d = wl.make_inputs_f8(L)
    kw = dict(cin=L.cin, kh=L.kh, kw=L.kw, korder=L.korder, stride=(2, 2), pad=(1, 1))
    sums = oracle.conv2d_f8(d["x"], d["W"], d["M"], **kw)
    scale = np.linspace(0.5, 2.0, L.cout).astype(np.float32)
    z = sums * scale.astype(np.float64) + d["bias"].astype(np.float64)
    assert np.array_equal(oracle.conv2d_f8(d["x"], d["W"], d["M"], scale=scale, bias=d["bias"], **kw), z)
    full = oracle.conv2d_f8(d["x"], d["W"], d["M"], scale=scale, bias=d["bias"], act=wl.ACT_RELU, **kw)
    assert np.array_equal(full, np.maximum(z, 0))
    idx = np.random.default_rng(0).choice(full.size, size=97, replace=False)
    pts = oracle.conv2d_f8_points(d["x"], d["W"], d["M"], idx, scale=scale, bias=d["bias"], act=wl.ACT_RELU, **kw)
    assert np.array_equal(pts, full.reshape(-1)[idx])
    # closed form: all weights and activations 1.0 (0x38), 3x3 window with zero padding -> 9 / 6 / 4 per input channel
    x = np.full((1, 4, 4, 4), 0x38, dtype=np.uint8)
    W = np.full((1, 36), 0x38, dtype=np.uint8)
    y = oracle.conv2d_f8(x, W, None, cin=4, kh=3, kw=3, korder=wl.K_CRS, pad=(1, 1))
    assert y[0, 1, 1, 0] == 36 and y[0, 0, 1, 0] == 24 and y[0, 0, 0, 0] == 16


def test_input_cast_matches_format_rules():
    a = np.array([0.0, 1.0, 1.0625, 1.1875, 447.0, 500.0, -1e9, 2.0 ** -9, 2.0 ** -10, 0.3], dtype=np.float32)
    b = wl.to_e4m3(a)
    v = oracle.e4m3_to_double(b)
    # ties to even (1.0625 is halfway between 1.0 and 1.125 -> 1.0; 1.1875 halfway between 1.125 and 1.25 -> 1.25),
    # saturation at 448, smallest subnormal, half of it rounds to zero
    assert list(v[:9]) == [0.0, 1.0, 1.0, 1.25, 448.0, 448.0, -448.0, 2.0 ** -9, 0.0]
    assert abs(v[9] - 0.3) <= 0.3 * 2.0 ** -4
