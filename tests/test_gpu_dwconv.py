"""GPU parity of the depthwise convolution against the fp64 oracle (ragged widths, every supported kernel width, both
dtypes), a bit-exact small-integer case, and the ConvNeXt-T stage-1 shape on sampled outputs."""
import numpy as np
import pytest
import torch

import oracle
from helpers import check_close, dev_bits, host_bits
from paper_2411_00288_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _run(ss, xb, wb, bias, dtype, pad, act):
    b = None if bias is None else torch.from_numpy(bias).cuda()
    y = ss.ss_dwconv2d_fwd(dev_bits(xb, dtype), dev_bits(wb, dtype), b, pad, act)
    torch.cuda.synchronize()
    return y


@pytest.mark.parametrize("shape", [(2, 9, 13, 24, 7, 7, 3), (3, 6, 7, 8, 3, 3, 1), (1, 11, 5, 40, 5, 5, 2), (2, 8, 9, 16, 3, 7, 0),
                                   (1, 7, 7, 96, 7, 7, 3), (1, 4, 3, 8, 3, 3, 2)])
@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
def test_dwconv_matches_oracle(ss, shape, dtype):
    N, H, W, C, kh, kw, p = shape
    rng = np.random.Generator(np.random.PCG64(21))
    xb = wl.to_bits(rng.standard_normal((N, H, W, C), dtype=np.float32), dtype)
    wb = wl.to_bits(rng.standard_normal((kh, kw, C), dtype=np.float32) * np.float32((2.0 / (kh * kw)) ** 0.5), dtype)
    bias = (rng.standard_normal(C) * 0.1).astype(np.float32)
    for act in (wl.ACT_NONE, wl.ACT_RELU):
        ref = oracle.dwconv2d(xb, wb, dtype=dtype, bias=bias, pad=(p, p), act=act)
        check_close(_run(ss, xb, wb, bias, dtype, (p, p), act), ref, f"{shape} act {act}")
    ref = oracle.dwconv2d(xb, wb, dtype=dtype, bias=None, pad=(p, p))
    check_close(_run(ss, xb, wb, None, dtype, (p, p), wl.ACT_NONE), ref, f"{shape} no bias")


def test_dwconv_small_integers_are_bit_exact(ss):
    rng = np.random.Generator(np.random.PCG64(3))
    x = rng.integers(0, 3, size=(2, 10, 11, 16)).astype(np.float32)
    w = rng.integers(-1, 2, size=(7, 7, 16)).astype(np.float32)
    bias = rng.integers(-2, 3, size=16).astype(np.float32)
    for dtype in (wl.F16, wl.BF16):           # |sum| <= 2*49 + 2 = 100: exact in both types
        xb, wb = wl.to_bits(x, dtype), wl.to_bits(w, dtype)
        ref = oracle.dwconv2d(xb, wb, dtype=dtype, bias=bias, pad=(3, 3))
        y = _run(ss, xb, wb, bias, dtype, (3, 3), wl.ACT_NONE)
        assert np.array_equal(host_bits(y), wl.to_bits(ref.astype(np.float32), dtype))


def test_dwconv_convnext_stage1_shape_sampled(ss):
    N, H, W, C = 128, 56, 56, 96
    g = torch.Generator(device="cuda").manual_seed(1)
    x = torch.randn((N, H, W, C), generator=g, device="cuda").to(torch.bfloat16)
    w = (torch.randn((7, 7, C), generator=g, device="cuda") * (2.0 / 49) ** 0.5).to(torch.bfloat16)
    bias = torch.randn(C, generator=g, device="cuda") * 0.1
    y = ss.ss_dwconv2d_fwd(x, w, bias, (3, 3))
    torch.cuda.synchronize()
    # the oracle on a few whole images (first, middle, last) is cheap enough
    for n in (0, 61, 127):
        ref = oracle.dwconv2d(host_bits(x[n:n + 1]), host_bits(w), dtype=wl.BF16, bias=bias.cpu().numpy(), pad=(3, 3))
        check_close(y[n:n + 1], ref, f"image {n}")


def test_dwconv_argument_errors(ss):
    x = torch.zeros((1, 8, 8, 12), dtype=torch.float16, device="cuda")
    with pytest.raises(ss.SSError):
        ss.ss_dwconv2d_fwd(x, torch.zeros((3, 3, 12), dtype=torch.float16, device="cuda"))        # C % 8 != 0
    x = torch.zeros((1, 8, 8, 16), dtype=torch.float16, device="cuda")
    with pytest.raises(ss.SSError):
        ss.ss_dwconv2d_fwd(x, torch.zeros((3, 4, 16), dtype=torch.float16, device="cuda"))        # kernel width 4
    with pytest.raises(ss.SSError):
        ss.ss_dwconv2d_fwd(x, torch.zeros((3, 3, 16), dtype=torch.bfloat16, device="cuda"))       # dtype mismatch
