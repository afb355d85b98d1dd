"""GPU parity of the FP8 (OCP E4M3) precision point, through the C ABI."""

import numpy as np
import pytest
import torch

import oracle
from oracle import device_layout as dl
from paper_2411_00288_amd import workloads as wl
from helpers import check_close

pytestmark = pytest.mark.gpu

TILE_IDS = [0, 1, 2, 3, 4, 5]


def _L(N, H, W, cin, cout, k, s=1, p=0, korder=wl.K_RSC, act=wl.ACT_RELU, seed=0, mask="logits"):
    return wl.Layer(f"f8n{N}h{H}w{W}c{cin}o{cout}k{k}s{s}", N=N, H=H, W=W, cin=cin, cout=cout, kh=k, kw=k, stride=s, pad=p,
                    dtype=wl.F8, korder=korder, act=act, mask=mask, seed=seed)


def _desc(ss, L):
    return ss.make_desc(L.cout, L.cin, L.kh, L.kw, wl.F8, L.korder)


def _run(ss, L, d, sparse=True, scale=True, bias=True):
    desc = _desc(ss, L)
    W = torch.from_numpy(d["W"]).cuda()
    M = None if d["M"] is None else torch.from_numpy(d["M"]).cuda()
    x = torch.from_numpy(d["x"]).cuda()
    sc = torch.from_numpy(d["scale"]).cuda() if scale else None
    b = torch.from_numpy(d["bias"]).cuda() if bias else None
    if sparse:
        y = ss.ss_conv2d_q8_fwd(desc, x, ss.ss_mask_compress(desc, W, M), sc, b, (L.stride,) * 2, (L.pad,) * 2, L.act)
    else:
        y = ss.ss_conv2d_q8_dense_fwd(desc, x, ss.ss_dense_pack(desc, W, M), sc, b, (L.stride,) * 2, (L.pad,) * 2, L.act)
    torch.cuda.synchronize()
    return y


def _ref(L, d, scale=True, bias=True):
    return oracle.conv2d_f8(d["x"], d["W"], d["M"], cin=L.cin, kh=L.kh, kw=L.kw, korder=L.korder,
                            scale=d["scale"] if scale else None, bias=d["bias"] if bias else None,
                            stride=(L.stride,) * 2, pad=(L.pad,) * 2, act=L.act)


@pytest.mark.parametrize("shape", [(64, 64, 3, 3, wl.K_RSC), (40, 8, 3, 3, wl.K_CRS), (7, 4, 1, 1, wl.K_CRS), (130, 36, 3, 3, wl.K_RSC)])
def test_packed_bytes_match_oracle_bit_for_bit(ss, shape):
    """FP8 weights are packed as bytes, whatever they encode: NaN (0x7F, 0xFF), -0 (0x80) and subnormals survive."""
    cout, cin, kh, kw, korder = shape
    L = wl.Layer("t", N=1, H=4, W=4, cin=cin, cout=cout, kh=kh, kw=kw, dtype=wl.F8, korder=korder, mask="logits", seed=31)
    d = wl.make_inputs_f8(L)
    Wb = d["W"].copy()
    n = min(4, Wb.size)
    Wb.reshape(-1)[:n] = np.array([0x7F, 0x80, 0x01, 0xFF], dtype=np.uint8)[:n]
    desc = _desc(ss, L)
    assert ss.ss_packed_bytes(desc) == dl.packed_bytes8(cout, L.K)
    W, M = torch.from_numpy(Wb).cuda(), torch.from_numpy(d["M"]).cuda()
    packed = ss.ss_mask_compress(desc, W, M).cpu().numpy()
    vals, meta = oracle.compress8(Wb.view(np.int8), d["M"])
    expect = dl.tile8(vals, meta, cin=cin, kh=kh, kw=kw, korder=korder)
    expect[24:28] = np.frombuffer(np.uint32(wl.F8).tobytes(), dtype=np.uint8)      # header word 6 = dtype
    assert np.array_equal(packed, expect)
    back = ss.ss_mask_decompress(desc, torch.from_numpy(packed).cuda()).cpu().numpy()
    assert np.array_equal(back.view(np.uint8), np.where(d["M"] == 1, Wb, 0))
    dense = ss.ss_dense_pack(desc, W, M).cpu().numpy()
    expect_d = dl.tile_dense8(np.where(d["M"] == 1, Wb, 0).astype(np.uint8).view(np.int8), cin=cin, kh=kh, kw=kw, korder=korder)
    expect_d[24:28] = expect[24:28]
    assert np.array_equal(dense, expect_d)


SHAPES = [
    _L(3, 14, 14, 64, 300, 3, p=1),
    _L(2, 13, 11, 128, 200, 3, p=1, korder=wl.K_CRS, seed=6),   # the paper's flattening: byte transpose of the taps, 2 chunks of 64 channels
    _L(2, 12, 12, 64, 136, 2, s=2, korder=wl.K_CRS, seed=7),    # 2x2 stride 2 in the paper's flattening
    _L(2, 9, 10, 128, 200, 3, p=1, seed=4),         # long-reduction staging
    _L(2, 15, 13, 96, 136, 3, s=2, p=1),
    _L(3, 9, 11, 160, 264, 1, korder=wl.K_CRS),
    _L(2, 10, 10, 64, 130, 1),
    _L(2, 12, 12, 96, 200, 2, s=2),
    _L(1, 7, 7, 512, 520, 3, p=1, seed=5),
    _L(2, 11, 12, 48, 64, 5, p=2, seed=2),
]


@pytest.mark.parametrize("L", SHAPES, ids=lambda L: L.name)
def test_convolution_matches_oracle(ss, L):
    d = wl.make_inputs_f8(L)
    ref = _ref(L, d)
    check_close(_run(ss, L, d, sparse=True), ref, f"{L.name} sparse")
    check_close(_run(ss, L, d, sparse=False), ref, f"{L.name} dense")


@pytest.mark.parametrize("tile", TILE_IDS)
@pytest.mark.parametrize("L", SHAPES[:8], ids=lambda L: L.name)
def test_every_tile_shape_matches_oracle(ss, force_tile, L, tile):
    d = wl.make_inputs_f8(L)
    ref = _ref(L, d)
    force_tile(tile)
    check_close(_run(ss, L, d, sparse=True), ref, f"{L.name} sparse tile {tile}")
    check_close(_run(ss, L, d, sparse=False), ref, f"{L.name} dense tile {tile}")


@pytest.mark.parametrize("tile", TILE_IDS)
def test_small_integers_are_bit_exact(ss, force_tile, tile):
    """Operands in {-2..2} (exact in E4M3), no scale, bias or activation, |sum| <= 2048: no rounding anywhere, so the
    output must equal the oracle bit for bit."""
    L = _L(3, 10, 9, 64, 150, 3, p=1, act=wl.ACT_NONE)
    rng = np.random.Generator(np.random.PCG64(tile))
    d = {"W": wl.to_e4m3(rng.integers(-1, 2, size=(L.cout, L.K)).astype(np.float32)),
         "x": wl.to_e4m3(rng.integers(-2, 3, size=(L.N, L.H, L.W, L.cin)).astype(np.float32)),
         "M": wl.mask_from_logits(rng.standard_normal((L.cout, L.K // 4, 6), dtype=np.float32)),
         "scale": None, "bias": None}
    assert 2 * L.K // 2 <= 2048
    ref = _ref(L, d, scale=False, bias=False)
    force_tile(tile)
    for sparse in (True, False):
        y = _run(ss, L, d, sparse=sparse, scale=False, bias=False)
        assert np.array_equal(y.float().cpu().numpy().astype(np.float64), ref)


def test_full_size_layer_at_sampled_points(ss):
    L = wl.Layer("cfg1_f8", N=32, H=14, W=14, cin=256, cout=256, kh=3, kw=3, stride=1, pad=1, dtype=wl.F8,
                 korder=wl.K_RSC, act=wl.ACT_RELU, mask="logits", seed=0)
    d = wl.make_inputs_f8(L)
    idx = np.random.default_rng(1).choice(L.P * L.cout, size=4096, replace=False)
    ref = oracle.conv2d_f8_points(d["x"], d["W"], d["M"], idx, cin=L.cin, kh=3, kw=3, korder=L.korder, scale=d["scale"],
                                  bias=d["bias"], stride=(1, 1), pad=(1, 1), act=L.act)
    for sparse in (True, False):
        y = _run(ss, L, d, sparse=sparse).float().cpu().numpy().astype(np.float64).reshape(-1)[idx]
        assert (np.abs(y - ref) <= 1e-2 * (np.abs(ref) + 1)).all()
        assert np.linalg.norm(y - ref) <= 2e-3 * np.linalg.norm(ref)
    assert (ref > 0).mean() > 0.2


def test_nan_byte_propagates_and_wrong_descriptor_is_rejected(ss):
    L = _L(1, 6, 6, 64, 64, 1, act=wl.ACT_NONE)
    d = wl.make_inputs_f8(L)
    d["x"][0, 2, 3, 5] = 0x7F
    y = _run(ss, L, d, sparse=False).float().cpu().numpy()
    assert np.isnan(y[0, 2, 3, :]).all() and np.isfinite(np.delete(y.reshape(36, 64), 2 * 6 + 3, axis=0)).all()
    desc = _desc(ss, L)
    x16 = torch.zeros((1, 6, 6, 64), dtype=torch.float16, device="cuda")
    packed = ss.ss_mask_compress(desc, torch.from_numpy(d["W"]).cuda(), torch.from_numpy(d["M"]).cuda())
    with pytest.raises(ss.SSError):
        ss.ss_conv2d_fwd(desc, x16, packed)
