"""The activation-stationary pointwise kernel (a workgroup keeps its 64 pixels' activations in LDS and walks down the
output channels) against the oracle.

The library picks it for the channel-expanding 1x1 layers; here it is forced (`ss_debug_force_tile(13)`) on small
ragged problems, with one, two and three workgroups per pixel tile (`ss_debug_force_split`), with and without a residual,
on the 2:4 path and the dense twin."""
import numpy as np
import pytest
import torch

import oracle
from helpers import check_close, dev_bits, host_bits, layer_desc
from paper_2411_00288_amd import workloads as wl

pytestmark = pytest.mark.gpu

ROWS_TILE = 13


def _L(N, H, W, cin, cout, s=1, p=0, dtype=wl.F16, act=wl.ACT_RELU, seed=0):
    return wl.Layer(f"rows_n{N}h{H}w{W}c{cin}o{cout}s{s}p{p}d{dtype}a{act}", N=N, H=H, W=W, cin=cin, cout=cout, kh=1, kw=1,
                    stride=s, pad=p, dtype=dtype, act=act, mask="logits", seed=seed)


def _residual(L, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    return wl.to_bits(rng.standard_normal((L.N, L.Ho, L.Wo, L.cout), dtype=np.float32), L.dtype)


def _run(ss, L, d, res_bits, sparse):
    desc = layer_desc(ss, L)
    W, x = dev_bits(d["W"], L.dtype), dev_bits(d["x"], L.dtype)
    M = torch.from_numpy(d["M"]).cuda()
    b = torch.from_numpy(d["bias"]).cuda()
    r = None if res_bits is None else dev_bits(res_bits, L.dtype)
    st, pd = (L.stride,) * 2, (L.pad,) * 2
    if sparse:
        wbuf = ss.ss_mask_compress(desc, W, M)
        y = ss.ss_conv2d_fwd(desc, x, wbuf, b, st, pd, L.act) if r is None else ss.ss_conv2d_res_fwd(desc, x, wbuf, b, r, st, pd, L.act)
    else:
        wbuf = ss.ss_dense_pack(desc, W, M)
        y = ss.ss_conv2d_dense_fwd(desc, x, wbuf, b, st, pd, L.act) if r is None else ss.ss_conv2d_dense_res_fwd(desc, x, wbuf, b, r, st, pd, L.act)
    torch.cuda.synchronize()
    return y


def _ref(L, d, res_bits):
    return oracle.conv2d(d["x"], d["W"], d["M"], cin=L.cin, kh=1, kw=1, korder=L.korder, dtype=L.dtype, bias=d["bias"],
                         stride=(L.stride,) * 2, pad=(L.pad,) * 2, act=L.act, residual=res_bits)


SHAPES = [
    _L(3, 9, 11, 64, 520),                                        # 297 pixels (ragged), 9 row blocks, the last with 8 channels
    _L(2, 14, 14, 128, 512, dtype=wl.BF16, act=wl.ACT_NONE, seed=1),      # 8 full row blocks
    _L(2, 15, 13, 256, 1024, s=2, dtype=wl.BF16, seed=2),         # stride 2: 8 x 7 outputs per image
    _L(1, 7, 7, 512, 2048, act=wl.ACT_GELU, seed=3),              # the longest reduction, 32 row blocks, 49 pixels
    _L(2, 6, 5, 64, 72, p=1, seed=4),                             # padding around a 1x1 kernel: border outputs see only the bias
    _L(5, 4, 4, 128, 200, dtype=wl.BF16, seed=5),                 # 80 pixels: a full and a quarter pixel tile; odd number of row tiles
    _L(2, 9, 9, 96, 384, dtype=wl.BF16, act=wl.ACT_GELU, seed=6), # an odd number of reduction steps, six row blocks over four waves
]


@pytest.mark.parametrize("groups", [None, 1, 2, 3])
@pytest.mark.parametrize("L", SHAPES, ids=lambda L: L.name)
def test_rows_kernel_matches_oracle(ss, force_tile, force_split, L, groups):
    force_tile(ROWS_TILE)
    force_split(groups)
    d = wl.make_inputs(L)
    ref = _ref(L, d, None)
    check_close(_run(ss, L, d, None, sparse=True), ref, f"{L.name} sparse")
    check_close(_run(ss, L, d, None, sparse=False), ref, f"{L.name} dense")


@pytest.mark.parametrize("L", SHAPES[:4], ids=lambda L: L.name)
def test_rows_kernel_with_residual(ss, force_tile, L):
    force_tile(ROWS_TILE)
    d = wl.make_inputs(L)
    res = _residual(L, 23)
    ref = _ref(L, d, res)
    check_close(_run(ss, L, d, res, sparse=True), ref, f"{L.name} sparse + residual")
    check_close(_run(ss, L, d, res, sparse=False), ref, f"{L.name} dense + residual")


@pytest.mark.parametrize("cin", [64, 256])
def test_rows_kernel_is_bit_exact_on_integers_and_equals_the_general_kernel(ss, force_tile, force_split, cin):
    L = _L(2, 9, 8, cin, 264, act=wl.ACT_NONE, seed=9)
    d = wl.make_small_int_inputs(L, seed=3)
    ref = _ref(L, d, None)
    force_tile(ROWS_TILE)
    force_split(2)
    y = _run(ss, L, d, None, sparse=True)
    assert np.array_equal(y.float().cpu().numpy().astype(np.float64), ref)
    yd = _run(ss, L, d, None, sparse=False)
    assert np.array_equal(yd.float().cpu().numpy().astype(np.float64), ref)
    force_tile(2)
    force_split(None)
    assert np.array_equal(host_bits(_run(ss, L, d, None, sparse=True)), host_bits(y))


def test_rows_kernel_in_hip_graph_replays_correctly(ss):
    """The library's own choice for a channel-expanding layer, with a residual tail, recorded twice in a HIP graph and
    replayed on changing inputs with eager work in between: every replay equals the eager result bit for bit."""
    L = _L(2, 14, 14, 128, 512, dtype=wl.BF16, seed=31)
    d = wl.make_inputs(L)
    desc = layer_desc(ss, L)
    x = dev_bits(d["x"], L.dtype)
    packed = ss.ss_mask_compress(desc, dev_bits(d["W"], L.dtype), torch.from_numpy(d["M"]).cuda())
    bias = torch.from_numpy(d["bias"]).cuda()
    res = dev_bits(_residual(L, 5), L.dtype)
    launch, y = ss.prepare_conv2d(desc, x, packed, bias, (1, 1), (0, 0), L.act, residual=res)
    launch()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            launch()
            launch()
    torch.cuda.synchronize()
    for rep in range(3):
        x.copy_(torch.roll(x, shifts=rep + 1, dims=2))          # new contents, same buffer
        eager = ss.ss_conv2d_res_fwd(desc, x, packed, bias, res, (1, 1), (0, 0), L.act)
        torch.cuda.synchronize()
        y.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), eager.view(torch.int16)), f"replay {rep}"
