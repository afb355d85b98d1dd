"""GPU parity of the weight compressor / decompressor / dense packer: bit-exact against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from oracle import device_layout as dl
from paper_2411_00288_amd import workloads as wl
from helpers import dev_bits, host_bits, layer_desc

pytestmark = pytest.mark.gpu

SHAPES = [  # cout, cin, kh, kw, korder
    (64, 64, 3, 3, wl.K_CRS),      # config-0 shape: K = 576 = 18 steps
    (256, 64, 1, 1, wl.K_CRS),
    (40, 8, 3, 3, wl.K_CRS),       # ragged rows (40 % 32), K = 72 (ragged step, odd step count)
    (7, 4, 1, 1, wl.K_CRS),        # a single block per row
    (96, 24, 2, 2, wl.K_RSC),      # K = 96 = 3 steps (odd: padded metadata half)
    (33, 96, 1, 1, wl.K_CRS),
    (130, 36, 3, 3, wl.K_RSC),     # K = 324: K % 32 = 4
    (1, 4, 1, 1, wl.K_CRS),
]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
@pytest.mark.parametrize("mask", ["logits", "top2"])
def test_packed_bytes_match_oracle_bit_for_bit(ss, shape, dtype, mask):
    cout, cin, kh, kw, korder = shape
    L = wl.Layer("t", N=1, H=4, W=4, cin=cin, cout=cout, kh=kh, kw=kw, dtype=dtype, korder=korder, mask=mask, seed=31)
    d = wl.make_inputs(L)
    Wb = d["W"].copy()
    special = [0x8000, 0x7E01, 0x7C00, 0x0001, 0xFC00, 0x8001, 0x0000, 0xFFFF]   # -0, NaN, inf, subnormals
    n = min(8, Wb.size)
    Wb.reshape(-1)[:n] = special[:n]
    desc = layer_desc(ss, L)
    assert ss.ss_packed_bytes(desc) == dl.packed_bytes(cout, L.K)
    W = dev_bits(Wb, dtype)
    M = torch.from_numpy(d["M"]).cuda()
    W_before, M_before = W.clone(), M.clone()
    packed = ss.ss_mask_compress(desc, W, M)
    vals, meta = oracle.compress(Wb, d["M"])
    expect = dl.tile(vals, meta, cin=cin, kh=kh, kw=kw, dtype=dtype, korder=korder)
    got = packed.cpu().numpy()
    assert got.size == expect.size
    assert np.array_equal(got, expect)
    # the inverse bijection recovers the canonical arrays from the GPU's bytes
    h, v2, m2 = dl.untile(got)
    assert np.array_equal(v2, vals) and np.array_equal(m2, meta)
    # inputs are never written (the original weights stay unchanged)
    assert torch.equal(W.view(torch.int16), W_before.view(torch.int16)) and torch.equal(M, M_before)
    # decompress gives M (.) W bit for bit, including the sign of kept zeros and NaN payloads
    back = host_bits(ss.ss_mask_decompress(desc, packed))
    assert np.array_equal(back, np.where(d["M"] == 1, Wb, 0).astype(np.uint16))
    assert np.array_equal(back, oracle.decompress(vals, meta))


def test_compress_reports_first_invalid_block(ss):
    L = wl.Layer("t", N=1, H=2, W=2, cin=16, cout=70, kh=3, kw=3, mask="logits", seed=1)
    d = wl.make_inputs(L)
    desc = layer_desc(ss, L)
    W = dev_bits(d["W"], L.dtype)
    for bad in ([(5, 7)], [(69, 35), (12, 0)], [(0, 0)], [(33, 20), (33, 3), (40, 1)]):
        Mb = d["M"].copy()
        for (r, g) in bad:
            Mb[r, 4 * g:4 * g + 4] = [1, 1, 1, 0]
        st, r0, g0 = oracle.mask_check(Mb)
        assert st == 1
        with pytest.raises(ss.SSError) as ei:
            ss.ss_mask_compress(desc, W, torch.from_numpy(Mb).cuda())
        assert ei.value.status == ss.SS_ERR_BAD_MASK
        assert ei.value.detail == (r0, g0) == min(bad)
    # a byte that is neither 0 nor 1 is rejected too
    Mb = d["M"].copy()
    Mb[3, 8:12] = [2, 0, 0, 0]
    with pytest.raises(ss.SSError) as ei:
        ss.ss_mask_compress(desc, W, torch.from_numpy(Mb).cuda())
    assert ei.value.detail == (3, 2)
    # all-zero and all-one blocks
    for fill in (0, 1):
        Mb = d["M"].copy()
        Mb[10, 0:4] = fill
        with pytest.raises(ss.SSError):
            ss.ss_mask_compress(desc, W, torch.from_numpy(Mb).cuda())


@pytest.mark.parametrize("shape", SHAPES + [(64, 3, 7, 7, wl.K_CRS), (5, 3, 3, 3, wl.K_RSC)])
@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
def test_dense_pack_matches_oracle_layout(ss, shape, dtype):
    cout, cin, kh, kw, korder = shape
    K = cin * kh * kw
    masked = K % 4 == 0
    L = wl.Layer("t", N=1, H=8, W=8, cin=cin, cout=cout, kh=kh, kw=kw, dtype=dtype, korder=korder,
                 mask="logits" if masked else "none", seed=17)
    d = wl.make_inputs(L)
    desc = layer_desc(ss, L)
    assert ss.ss_dense_bytes(desc) == dl.dense_bytes(cout, K)
    W = dev_bits(d["W"], dtype)
    M = torch.from_numpy(d["M"]).cuda() if masked else None
    got = ss.ss_dense_pack(desc, W, M).cpu().numpy()
    Wm = np.where(d["M"] == 1, d["W"], 0).astype(np.uint16) if masked else d["W"]
    expect = dl.tile_dense(Wm, cin=cin, kh=kh, kw=kw, dtype=dtype, korder=korder)
    assert np.array_equal(got, expect)


def test_full_size_config1_compress(ss):
    L = wl.CONFIG1
    d = wl.make_inputs(wl.with_batch(L, 1))
    desc = layer_desc(ss, L)
    packed = ss.ss_mask_compress(desc, dev_bits(d["W"], L.dtype), torch.from_numpy(d["M"]).cuda())
    vals, meta = oracle.compress(d["W"], d["M"])
    expect = dl.tile(vals, meta, cin=L.cin, kh=L.kh, kw=L.kw, dtype=L.dtype, korder=L.korder)
    assert np.array_equal(packed.cpu().numpy(), expect)
    assert packed.numel() == 256 + 9 * (L.cout * L.K * 2) // 16


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
def test_update_and_repack_match_oracle_bit_for_bit(ss, shape, dtype):
    """W <- round16(W + U), packed <- compress(W, M): both bit for bit (values chosen without NaN results)."""
    cout, cin, kh, kw, korder = shape
    L = wl.Layer("t", N=1, H=4, W=4, cin=cin, cout=cout, kh=kh, kw=kw, dtype=dtype, korder=korder, mask="logits", seed=41)
    d = wl.make_inputs(L)
    rng = np.random.Generator(np.random.PCG64(7))
    scale = np.float32(2.0 ** rng.integers(-12, 3, size=d["W"].shape))     # updates from far below an ulp to larger than W
    Ub = wl.to_bits(rng.standard_normal(d["W"].shape, dtype=np.float32) * scale, dtype)
    Wb = d["W"].copy()
    edge = [(0x0001, 0x0001), (0x8000, 0x0000), (0x7BFF if dtype == wl.F16 else 0x7F7F, 0x7BFF if dtype == wl.F16 else 0x7F7F),
            (0x3C00, 0xBC00), (0x03FF, 0x0001)]
    for i, (a, b) in enumerate(edge[:min(len(edge), Wb.size)]):
        Wb.reshape(-1)[i], Ub.reshape(-1)[i] = a, b
    V = oracle.update(Wb, Ub, dtype)
    desc = layer_desc(ss, L)
    W, U, M = dev_bits(Wb, dtype), dev_bits(Ub, dtype), torch.from_numpy(d["M"]).cuda()
    U_before = U.clone()
    packed = ss.ss_mask_update_compress(desc, W, U, M)
    assert np.array_equal(host_bits(W), V)
    assert torch.equal(U.view(torch.int16), U_before.view(torch.int16))
    vals, meta = oracle.compress(V, d["M"])
    assert np.array_equal(packed.cpu().numpy(), dl.tile(vals, meta, cin=cin, kh=kh, kw=kw, dtype=dtype, korder=korder))
    # the same bytes as packing the updated weights from scratch
    assert torch.equal(packed, ss.ss_mask_compress(desc, W, M))


def test_convolution_after_an_update_uses_the_new_weights(ss):
    L = wl.Layer("t", N=2, H=9, W=9, cin=64, cout=96, kh=3, kw=3, stride=1, pad=1, dtype=wl.BF16, act=wl.ACT_RELU,
                 mask="logits", seed=12)
    d = wl.make_inputs(L)
    rng = np.random.Generator(np.random.PCG64(8))
    Ub = wl.to_bits(rng.standard_normal(d["W"].shape, dtype=np.float32) * np.float32(0.05), L.dtype)
    desc = layer_desc(ss, L)
    W, U, M = dev_bits(d["W"], L.dtype), dev_bits(Ub, L.dtype), torch.from_numpy(d["M"]).cuda()
    packed = ss.ss_mask_update_compress(desc, W, U, M)
    y = ss.ss_conv2d_fwd(desc, dev_bits(d["x"], L.dtype), packed, torch.from_numpy(d["bias"]).cuda(), (1, 1), (1, 1), L.act)
    V = oracle.update(d["W"], Ub, L.dtype)
    ref = oracle.conv2d(d["x"], V, d["M"], cin=L.cin, kh=3, kw=3, dtype=L.dtype, bias=d["bias"], pad=(1, 1), act=L.act)
    from helpers import check_close
    check_close(y, ref, "conv after update")
    old = oracle.conv2d(d["x"], d["W"], d["M"], cin=L.cin, kh=3, kw=3, dtype=L.dtype, bias=d["bias"], pad=(1, 1), act=L.act)
    assert np.linalg.norm(ref - old) / np.linalg.norm(old) > 0.05          # the update is visible at this tolerance


def test_update_compress_argument_and_mask_errors(ss):
    L = wl.Layer("t", N=1, H=2, W=2, cin=16, cout=40, kh=1, kw=1, mask="logits", seed=1)
    d = wl.make_inputs(L)
    desc = layer_desc(ss, L)
    W, M = dev_bits(d["W"], L.dtype), torch.from_numpy(d["M"]).cuda()
    with pytest.raises(ss.SSError):
        ss.ss_mask_update_compress(desc, W, W[:10], M)
    Mb = d["M"].copy()
    Mb[3, 4:8] = [1, 1, 1, 0]
    U = torch.zeros_like(W)
    with pytest.raises(ss.SSError) as e:
        ss.ss_mask_update_compress(desc, W, U, torch.from_numpy(Mb).cuda())
    assert e.value.status == ss.SS_ERR_BAD_MASK and e.value.detail == (3, 1)
