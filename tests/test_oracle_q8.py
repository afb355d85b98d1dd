"""Pins of the oracle's 8-bit integer functions (CPU only): each is checked against something other than itself."""
import itertools

import numpy as np
import pytest
import torch

import oracle
from oracle import device_layout as dl
from paper_2411_00288_amd import workloads as wl


def _layer(**kw):
    base = dict(name="t", N=2, H=6, W=5, cin=8, cout=6, kh=3, kw=3, stride=1, pad=1, dtype=wl.I8, korder=wl.K_RSC,
                mask="logits", seed=3)
    base.update(kw)
    return wl.Layer(**base)


def _unfold_matmul(x, Wm, L):
    """Eq. (5) written out in numpy with int64 arithmetic: explicit unfold, then one matrix product."""
    N, H, Wd, cin = x.shape
    xp = np.zeros((N, H + 2 * L.pad, Wd + 2 * L.pad, cin), dtype=np.int64)
    xp[:, L.pad:L.pad + H, L.pad:L.pad + Wd, :] = x
    cols = np.zeros((L.K, N * L.Ho * L.Wo), dtype=np.int64)
    for c, r, t in itertools.product(range(cin), range(L.kh), range(L.kw)):
        k = (c * L.kh + r) * L.kw + t if L.korder == wl.K_CRS else (r * L.kw + t) * cin + c
        patch = xp[:, r:r + L.stride * L.Ho:L.stride, t:t + L.stride * L.Wo:L.stride, c]
        cols[k] = patch.reshape(-1)
    return (Wm.astype(np.int64) @ cols).T.reshape(N, L.Ho, L.Wo, L.cout)


@pytest.mark.parametrize("korder", [wl.K_CRS, wl.K_RSC])
@pytest.mark.parametrize("geom", [dict(), dict(stride=2, pad=0), dict(kh=1, kw=1, pad=0, cin=12), dict(kh=2, kw=2, stride=2, pad=0)])
def test_integer_sums_equal_unfold_matmul(korder, geom):
    L = _layer(korder=korder, **geom)
    d = wl.make_inputs_q8(L)
    Wm = np.where(d["M"] == 1, d["W"], 0)
    ref = _unfold_matmul(d["x"], Wm, L)
    got = oracle.conv2d_q8(d["x"], d["W"], d["M"], cin=L.cin, kh=L.kh, kw=L.kw, korder=korder,
                           stride=(L.stride,) * 2, pad=(L.pad,) * 2)
    assert np.array_equal(got, ref.astype(np.float64))      # exact: |sum| is far below 2^53
    # M = None is the plain dense convolution
    got_d = oracle.conv2d_q8(d["x"], d["W"], None, cin=L.cin, kh=L.kh, kw=L.kw, korder=korder,
                             stride=(L.stride,) * 2, pad=(L.pad,) * 2)
    assert np.array_equal(got_d, _unfold_matmul(d["x"], d["W"], L).astype(np.float64))


def test_matches_a_float64_library_convolution():
    L = _layer(korder=wl.K_CRS, N=3, H=9, W=7, cin=4, cout=5, stride=2, pad=1)
    d = wl.make_inputs_q8(L)
    Wm = np.where(d["M"] == 1, d["W"], 0).astype(np.float64).reshape(L.cout, L.cin, L.kh, L.kw)
    xt = torch.from_numpy(d["x"].astype(np.float64)).permute(0, 3, 1, 2)
    ref = torch.nn.functional.conv2d(xt, torch.from_numpy(Wm), stride=L.stride, padding=L.pad).permute(0, 2, 3, 1).numpy()
    got = oracle.conv2d_q8(d["x"], d["W"], d["M"], cin=L.cin, kh=L.kh, kw=L.kw, korder=wl.K_CRS,
                           stride=(L.stride,) * 2, pad=(L.pad,) * 2)
    assert np.array_equal(got, ref)       # every product and partial sum is an integer below 2^53


def test_agrees_with_the_16_bit_oracle_on_the_same_integers():
    """Integers up to 127 are exact in binary16, and the fp64 sums of the 16-bit function are exact too."""
    L = _layer(korder=wl.K_RSC, act=wl.ACT_RELU)
    d = wl.make_inputs_q8(L)
    bias = d["bias"]
    ref = oracle.conv2d(wl.to_bits(d["x"].astype(np.float32), wl.F16), wl.to_bits(d["W"].astype(np.float32), wl.F16), d["M"],
                        cin=L.cin, kh=L.kh, kw=L.kw, korder=L.korder, dtype=wl.F16, bias=bias, stride=(1, 1), pad=(1, 1),
                        act=wl.ACT_RELU)
    got = oracle.conv2d_q8(d["x"], d["W"], d["M"], cin=L.cin, kh=L.kh, kw=L.kw, korder=L.korder, bias=bias,
                           stride=(1, 1), pad=(1, 1), act=wl.ACT_RELU)
    assert np.array_equal(got, ref)


def test_scale_bias_and_activation_follow_the_layer_model():
    L = _layer()
    d = wl.make_inputs_q8(L)
    kw = dict(cin=L.cin, kh=L.kh, kw=L.kw, korder=L.korder, stride=(1, 1), pad=(1, 1))
    sums = oracle.conv2d_q8(d["x"], d["W"], d["M"], **kw)
    scale = np.linspace(0.5, 2.0, L.cout).astype(np.float32)     # some not exactly representable in few bits
    bias = d["bias"]
    z = sums * scale.astype(np.float64) + bias.astype(np.float64)
    assert np.array_equal(oracle.conv2d_q8(d["x"], d["W"], d["M"], scale=scale, bias=bias, **kw), z)
    assert np.array_equal(oracle.conv2d_q8(d["x"], d["W"], d["M"], scale=scale, bias=bias, act=wl.ACT_RELU, **kw),
                          np.maximum(z, 0))
    g = oracle.conv2d_q8(d["x"], d["W"], d["M"], scale=scale, bias=bias, act=wl.ACT_GELU, **kw)
    phi = 0.5 * (1.0 + torch.erf(torch.from_numpy(z) / np.sqrt(2.0)).numpy())
    assert np.allclose(g, z * phi, rtol=1e-13, atol=1e-15)
    # extreme operands: -128 * -128 summed over the whole window, no wrap-around anywhere
    x = np.full((1, 3, 3, 4), -128, dtype=np.int8)
    W = np.full((1, 36), -128, dtype=np.int8)
    y = oracle.conv2d_q8(x, W, None, cin=4, kh=3, kw=3, korder=wl.K_CRS, pad=(1, 1))
    assert y[0, 1, 1, 0] == 36 * 16384 and y[0, 0, 0, 0] == 16 * 16384


def test_sampled_points_equal_the_full_tensor():
    L = _layer(N=2, H=7, W=7, cin=8, cout=10, stride=2)
    d = wl.make_inputs_q8(L)
    kw = dict(cin=L.cin, kh=L.kh, kw=L.kw, korder=L.korder, scale=d["scale"], bias=d["bias"], stride=(2, 2),
              pad=(1, 1), act=wl.ACT_RELU)
    full = oracle.conv2d_q8(d["x"], d["W"], d["M"], **kw)
    idx = np.random.default_rng(0).choice(full.size, size=97, replace=False)
    assert np.array_equal(oracle.conv2d_q8_points(d["x"], d["W"], d["M"], idx, **kw), full.reshape(-1)[idx])


def test_representation_brute_force_over_the_six_patterns():
    W = np.array([[-5, 7, 0, -128]], dtype=np.int8)
    seen = set()
    for pat in wl.PATTERNS:
        vals, meta = oracle.compress8(W, pat[None, :])
        kept = [i for i in range(4) if pat[i]]
        assert list(vals[0]) == [W[0, kept[0]], W[0, kept[1]]]
        assert meta[0, 0] == kept[0] | (kept[1] << 2)
        assert np.array_equal(oracle.decompress8(vals, meta), np.where(pat == 1, W, 0))
        seen.add(int(meta[0, 0]))
    assert len(seen) == 6
    for bad in ([1, 1, 1, 0], [1, 0, 0, 0], [2, 1, 0, 0]):
        with pytest.raises(ValueError):
            oracle.compress8(W, np.array([bad], dtype=np.uint8))


@pytest.mark.parametrize("shape", [(40, 8, 3, 3), (7, 4, 1, 1), (96, 24, 2, 2), (33, 96, 1, 1), (130, 36, 3, 3), (1, 4, 1, 1)])
def test_round_trip_and_device_layout_bijection(shape):
    cout, cin, kh, kw = shape
    L = _layer(cout=cout, cin=cin, kh=kh, kw=kw, N=1, H=4, W=4)
    d = wl.make_inputs_q8(L)
    vals, meta = oracle.compress8(d["W"], d["M"])
    assert vals.shape == (cout, L.K // 2) and meta.shape == (cout, L.K // 4)
    assert np.array_equal(oracle.decompress8(vals, meta), np.where(d["M"] == 1, d["W"], 0))
    # the kept positions are the mask's ones, in ascending order
    pos = np.stack([meta & 3, (meta >> 2) & 3], axis=-1)
    assert (pos[..., 0] < pos[..., 1]).all()
    rebuilt = np.zeros((cout, L.K // 4, 4), dtype=np.uint8)
    np.put_along_axis(rebuilt, pos.astype(np.int64), 1, axis=-1)
    assert np.array_equal(rebuilt.reshape(cout, L.K), d["M"])
    # device permutation: a bijection of the canonical arrays, padding included in the byte count
    packed = dl.tile8(vals, meta, cin=cin, kh=kh, kw=kw, korder=L.korder)
    assert packed.size == dl.packed_bytes8(cout, L.K) == 256 + (-(-cout // 32)) * (-(-L.K // 64)) * 1280
    h, v2, m2 = dl.untile8(packed)
    assert np.array_equal(v2, vals) and np.array_equal(m2, meta)
    assert list(h[:10]) == [dl.MAGIC_SPARSE, 1, cout, cin, kh, kw, 2, L.korder, -(-cout // 32), -(-L.K // 64)]
    # every canonical byte appears exactly once among the non-padding slots: tiling a ramp shows the permutation
    ramp = (np.arange(cout * (L.K // 2)) % 251 + 1).astype(np.uint8).view(np.int8).reshape(cout, L.K // 2)
    body = dl.tile8(ramp, meta, cin=cin, kh=kh, kw=kw, korder=L.korder)[256:256 + (-(-cout // 32)) * (-(-L.K // 64)) * 1024]
    assert np.count_nonzero(body) == ramp.size
    assert np.array_equal(np.sort(body[body != 0]), np.sort(ramp.view(np.uint8).reshape(-1)))


def test_dense_twin_layout_places_every_element_once():
    cout, cin, kh, kw = 40, 12, 3, 3
    K = cin * kh * kw
    Wm = (np.arange(cout * K) % 127 + 1).astype(np.int8).reshape(cout, K)
    out = dl.tile_dense8(Wm, cin=cin, kh=kh, kw=kw, korder=wl.K_RSC)
    assert out.size == dl.dense_bytes8(cout, K)
    body = out[256:].reshape(-(-cout // 32), -(-K // 64), 2, 64, 16)
    assert np.count_nonzero(body) == cout * K
    # spot positions from the stated rule: tile (mt, ks, h), lane l, slot s <-> row 32 mt + l%32, k = 64 ks + 32 (l//32) + 16 h + s
    for (mt, ks, h, l, s) in [(0, 0, 0, 0, 0), (1, 1, 1, 39, 5), (0, 1, 0, 63, 15), (1, 0, 1, 7, 9)]:
        row, k = 32 * mt + l % 32, 64 * ks + 32 * (l // 32) + 16 * h + s
        expect = Wm[row, k] if row < cout and k < K else 0
        assert body[mt, ks, h, l, s] == np.uint8(expect)
