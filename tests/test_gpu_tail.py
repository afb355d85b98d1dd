"""GPU parity of the fused layer tail through the C ABI: y = act(conv + bias + residual), act in {none, ReLU, GELU}.

Checked against the fp64 oracle element by element (every tile shape, both paths, ragged sizes), bit for bit on
small-integer inputs, in place (y aliasing the residual), and at full size on a ResNet-50 conv3 layer (sampled
outputs) in the launch configuration the benchmark uses.
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from helpers import check_close, dev_bits, host_bits, layer_desc
from paper_2411_00288_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _L(N, H, W, cin, cout, k, s=1, p=0, dtype=wl.F16, korder=wl.K_CRS, act=wl.ACT_RELU, seed=0):
    return wl.Layer(f"n{N}h{H}w{W}c{cin}o{cout}k{k}s{s}d{dtype}a{act}", N=N, H=H, W=W, cin=cin, cout=cout, kh=k, kw=k,
                    stride=s, pad=p, dtype=dtype, korder=korder, act=act, mask="logits", seed=seed)


def _residual(L, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    Ho, Wo = (L.H + 2 * L.pad - L.kh) // L.stride + 1, (L.W + 2 * L.pad - L.kw) // L.stride + 1
    return wl.to_bits(rng.standard_normal((L.N, Ho, Wo, L.cout), dtype=np.float32), L.dtype)


def _run(ss, L, d, res_bits, sparse=True, in_place=False):
    desc = layer_desc(ss, L)
    W, x = dev_bits(d["W"], L.dtype), dev_bits(d["x"], L.dtype)
    M = torch.from_numpy(d["M"]).cuda()
    b = torch.from_numpy(d["bias"]).cuda()
    r = None if res_bits is None else dev_bits(res_bits, L.dtype)
    y = r if in_place else None
    if sparse:
        wbuf = ss.ss_mask_compress(desc, W, M)
        y = ss.ss_conv2d_res_fwd(desc, x, wbuf, b, r, (L.stride,) * 2, (L.pad,) * 2, L.act, y=y)
    else:
        wbuf = ss.ss_dense_pack(desc, W, M)
        y = ss.ss_conv2d_dense_res_fwd(desc, x, wbuf, b, r, (L.stride,) * 2, (L.pad,) * 2, L.act, y=y)
    torch.cuda.synchronize()
    return y


def _ref(L, d, res_bits):
    return oracle.conv2d(d["x"], d["W"], d["M"], cin=L.cin, kh=L.kh, kw=L.kw, korder=L.korder, dtype=L.dtype,
                         bias=d["bias"], stride=(L.stride,) * 2, pad=(L.pad,) * 2, act=L.act, residual=res_bits)


SHAPES = [
    _L(3, 14, 14, 64, 300, 3, p=1),                                   # tap transpose, ragged rows and pixels
    _L(2, 15, 13, 96, 136, 3, s=2, p=1, dtype=wl.BF16, act=wl.ACT_NONE),
    _L(3, 9, 11, 160, 264, 1, dtype=wl.BF16),                         # pointwise, ragged everything
    _L(2, 10, 10, 64, 130, 1, act=wl.ACT_GELU),                       # cout % 8 != 0: scalar store path
    _L(2, 12, 12, 96, 200, 2, s=2, act=wl.ACT_GELU, dtype=wl.BF16),
    _L(1, 11, 9, 12, 150, 3, p=1),                                    # gather fallback, cout % 8 != 0
]


@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4, 5])
@pytest.mark.parametrize("L", SHAPES, ids=lambda L: L.name)
def test_residual_tail_matches_oracle_on_every_tile(ss, force_tile, L, tile):
    force_tile(tile)
    d = wl.make_inputs(L)
    res = _residual(L, 17)
    ref = _ref(L, d, res)
    check_close(_run(ss, L, d, res, sparse=True), ref, f"{L.name} tile {tile} sparse")
    check_close(_run(ss, L, d, res, sparse=False), ref, f"{L.name} tile {tile} dense")


@pytest.mark.parametrize("act", [wl.ACT_NONE, wl.ACT_RELU, wl.ACT_GELU])
def test_activations_without_residual_through_both_entry_points(ss, act):
    L = _L(2, 9, 9, 64, 72, 3, p=1, act=act, dtype=wl.BF16)
    d = wl.make_inputs(L)
    ref = _ref(L, d, None)
    check_close(_run(ss, L, d, None, sparse=True), ref, "res entry, no residual")
    desc = layer_desc(ss, L)
    wbuf = ss.ss_mask_compress(desc, dev_bits(d["W"], L.dtype), torch.from_numpy(d["M"]).cuda())
    y = ss.ss_conv2d_fwd(desc, dev_bits(d["x"], L.dtype), wbuf, torch.from_numpy(d["bias"]).cuda(), (1, 1), (1, 1), act)
    check_close(y, ref, "plain entry")


@pytest.mark.parametrize("sparse", [True, False])
@pytest.mark.parametrize("L", [_L(2, 7, 6, 32, 40, 3, p=1), _L(3, 9, 9, 64, 72, 1, act=wl.ACT_NONE),
                               _L(1, 9, 8, 16, 24, 3, s=2, p=1, dtype=wl.BF16)], ids=lambda L: L.name)
def test_small_integer_inputs_with_residual_are_bit_exact(ss, L, sparse):
    # integers small enough that neither the sum nor the residual add is ever rounded
    assert L.K + 2 + 8 <= (2048 if L.dtype == wl.F16 else 256)
    d = wl.make_small_int_inputs(L, seed=5)
    rng = np.random.Generator(np.random.PCG64(9))
    Ho, Wo = (L.H + 2 * L.pad - L.kh) // L.stride + 1, (L.W + 2 * L.pad - L.kw) // L.stride + 1
    res = wl.to_bits(rng.integers(-8, 9, size=(L.N, Ho, Wo, L.cout)).astype(np.float32), L.dtype)
    y = _run(ss, L, d, res, sparse=sparse)
    ref = _ref(L, d, res)
    assert np.array_equal(host_bits(y), wl.to_bits(ref.astype(np.float32), L.dtype))


def test_output_may_alias_the_residual(ss):
    L = _L(2, 14, 14, 64, 256, 1, dtype=wl.BF16)
    d = wl.make_inputs(L)
    res = _residual(L, 3)
    ref = _ref(L, d, res)
    y_sep = _run(ss, L, d, res)
    y_inp = _run(ss, L, d, res, in_place=True)
    check_close(y_inp, ref, "in place")
    assert torch.equal(y_sep.view(torch.int16), y_inp.view(torch.int16))


def test_argument_errors_of_the_residual_entry(ss):
    L = _L(1, 6, 6, 32, 32, 1)
    d = wl.make_inputs(L)
    desc = layer_desc(ss, L)
    x = dev_bits(d["x"], L.dtype)
    wbuf = ss.ss_mask_compress(desc, dev_bits(d["W"], L.dtype), torch.from_numpy(d["M"]).cuda())
    bad = torch.zeros((1, 6, 6, 16), dtype=torch.float16, device="cuda")
    with pytest.raises(ss.SSError):
        ss.ss_conv2d_res_fwd(desc, x, wbuf, None, bad)
    with pytest.raises(ss.SSError):
        ss.ss_conv2d_res_fwd(desc, x, wbuf, None, None, act=3)


def test_resnet_conv3_tail_full_size_sampled(ss):
    # 64 -> 256 1x1 at 56x56, batch 64: the last conv of a stage-1 bottleneck, closed by add + ReLU
    L = [l for l in wl.resnet50_layers() if l.name == "s1_c3_1x1_64_256"][0]
    L = dataclasses.replace(L, act=wl.ACT_RELU)
    d = wl.make_inputs(L)
    res = _residual(L, 23)
    y = _run(ss, L, d, res)
    rng = np.random.Generator(np.random.PCG64(1))
    idx = np.sort(rng.choice(y.numel(), size=20000, replace=False))
    ref = oracle.conv2d_points(d["x"], d["W"], d["M"], idx, cin=L.cin, kh=1, kw=1, dtype=L.dtype, bias=d["bias"],
                               act=L.act, residual=res)
    got = y.reshape(-1)[torch.from_numpy(idx).cuda()].float().cpu().numpy().astype(np.float64)
    assert np.linalg.norm(got - ref) / np.linalg.norm(ref) <= 2e-3
    assert (np.abs(got - ref) <= 1e-2 * (np.abs(ref) + 1)).all()


def test_gelu_over_a_dense_grid_of_arguments(ss):
    # zero weights: the pre-activation is the residual, here every fp16 value with |z| <= 16 (both signs), so the
    # kernel's normal-CDF evaluation is compared with the oracle's erf over its whole useful range
    pats = np.arange(0, 0x4C01, dtype=np.uint16)                     # +0 .. 16.0
    z_bits = np.concatenate([pats, pats | 0x8000])
    C = 64
    n = (z_bits.size + C - 1) // C
    z_bits = np.concatenate([z_bits, np.zeros(n * C - z_bits.size, dtype=np.uint16)]).reshape(1, n, 1, C)
    L = wl.Layer("gelu_grid", N=1, H=n, W=1, cin=32, cout=C, kh=1, kw=1, dtype=wl.F16, act=wl.ACT_GELU, mask="logits")
    d = wl.make_inputs(L)
    d["W"] = np.zeros_like(d["W"])
    d["bias"] = np.zeros_like(d["bias"])
    ref = _ref(L, d, z_bits)
    for sparse in (True, False):
        got = _run(ss, L, d, z_bits, sparse=sparse).float().cpu().numpy().astype(np.float64)
        assert (np.abs(got - ref) <= 1e-3 * np.abs(ref) + 1e-6).all()
