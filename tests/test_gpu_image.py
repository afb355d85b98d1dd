"""The dense 7x7 stride-2 first-layer kernel (an image of 3 or 4 channels) against the oracle.

The library picks it by itself for every such layer on the dense path; the tests also cap the number of resident
workgroups (`ss_debug_limit_blocks`) so that one workgroup walks over several output tiles, and compare with the
general kernel (a forced tile shape switches the image kernel off)."""
import numpy as np
import pytest
import torch

from paper_2411_00288_amd import workloads as wl
from helpers import check_close, dev_bits, host_bits, layer_desc, oracle_ref, run_gpu

pytestmark = pytest.mark.gpu


def _L(N, H, W, cin, cout, pad=3, dtype=wl.F16, korder=wl.K_CRS, act=wl.ACT_RELU, seed=0):
    return wl.Layer(f"img_n{N}h{H}w{W}c{cin}o{cout}p{pad}d{dtype}k{korder}a{act}", N=N, H=H, W=W, cin=cin, cout=cout, kh=7, kw=7,
                    stride=2, pad=pad, dtype=dtype, korder=korder, act=act, mask="none", relu_input=False, seed=seed)


SHAPES = [
    _L(2, 64, 64, 3, 64),                                                   # 32 x 32 outputs: 2 x 2 full tiles per image
    _L(3, 37, 45, 3, 64, dtype=wl.BF16, korder=wl.K_RSC, seed=1),           # 19 x 23 outputs: ragged tiles in both directions
    _L(2, 40, 70, 4, 64, korder=wl.K_RSC, act=wl.ACT_NONE, seed=2),         # four-channel image, channels-last flattening
    _L(1, 51, 33, 4, 72, dtype=wl.BF16, act=wl.ACT_GELU, seed=3),           # two channel groups, the second with 8 channels
    _L(2, 33, 35, 3, 24, pad=0, seed=4),                                    # no padding, fewer than 32 output channels
    _L(1, 20, 18, 4, 128, pad=5, dtype=wl.BF16, seed=5),                    # more padding than the kernel's half width
    _L(5, 7, 9, 3, 64, pad=0, korder=wl.K_RSC, seed=6),                     # kernel as large as the image: one output row
]


@pytest.mark.parametrize("cap", [None, 1, 3])
@pytest.mark.parametrize("L", SHAPES, ids=lambda L: L.name)
def test_image_kernel_matches_oracle(ss, limit_blocks, L, cap):
    d = wl.make_inputs(L)
    limit_blocks(cap)
    y = run_gpu(ss, L, d, sparse=False)
    check_close(y.reshape(L.N, L.Ho, L.Wo, L.cout), oracle_ref(L, d), L.name)


@pytest.mark.parametrize("cin", [3, 4])
@pytest.mark.parametrize("korder", [wl.K_CRS, wl.K_RSC])
def test_image_kernel_is_bit_exact_on_integers_and_equals_the_general_kernel(ss, force_tile, limit_blocks, cin, korder):
    L = _L(2, 45, 39, cin, 64, korder=korder, act=wl.ACT_NONE, seed=11)
    d = wl.make_small_int_inputs(L, seed=5)
    d["M"] = None                      # the layer is dense
    limit_blocks(2)
    y = run_gpu(ss, L, d, sparse=False)
    ref = oracle_ref(L, d)
    got = y.reshape(L.N, L.Ho, L.Wo, L.cout).float().cpu().numpy().astype(np.float64)
    assert np.array_equal(got, ref)
    force_tile(2)                      # a forced tile shape selects the general kernel
    y2 = run_gpu(ss, L, d, sparse=False)
    assert np.array_equal(host_bits(y2), host_bits(y))


def test_a_non_finite_pixel_reaches_exactly_the_windows_that_contain_it(ss):
    """Every window reads eight taps per kernel row from the shared patch, the eighth under a zero weight: a NaN or an
    infinity there must not leak into the window's sum."""
    L = _L(1, 48, 48, 3, 64, act=wl.ACT_NONE, seed=21)
    d = wl.make_inputs(L)
    x = d["x"].reshape(L.N, L.H, L.W, L.cin).copy()
    poison = [(10, 21, 0, 0x7E00), (30, 8, 2, 0x7C00)]          # (row, column, channel, bits): a NaN and +inf in binary16
    for (ih, iw, c, bits) in poison:
        x[0, ih, iw, c] = bits
    d["x"] = x.reshape(d["x"].shape)
    y = run_gpu(ss, L, d, sparse=False).reshape(L.N, L.Ho, L.Wo, L.cout).float().cpu().numpy()
    hit = np.zeros((L.Ho, L.Wo), dtype=bool)
    for (ih, iw, _, _) in poison:
        for ho in range(L.Ho):
            for wo in range(L.Wo):
                if 0 <= ih - (2 * ho - L.pad) < 7 and 0 <= iw - (2 * wo - L.pad) < 7:
                    hit[ho, wo] = True
    bad = ~np.isfinite(y).all(axis=-1)[0]
    # a window that contains the poisoned pixel is non-finite in at least one channel (its weight there is not zero);
    # a window that does not contain it is finite in every channel
    assert not (bad & ~hit).any(), np.argwhere(bad & ~hit)
    assert (np.isfinite(y[0]).any(axis=-1) | hit).all()
    assert (~np.isfinite(y[0])).any(axis=-1)[hit].all()


def test_image_kernel_in_hip_graph_replays_correctly(ss):
    """Recorded twice in a HIP graph and replayed on changing images with eager work in between: every replay equals
    the eager result bit for bit."""
    L = _L(2, 70, 66, 4, 64, korder=wl.K_RSC, dtype=wl.BF16, seed=33)
    d = wl.make_inputs(L)
    desc = layer_desc(ss, L)
    x = dev_bits(d["x"], L.dtype)
    wbuf = ss.ss_dense_pack(desc, dev_bits(d["W"], L.dtype), None)
    bias = torch.from_numpy(d["bias"]).cuda()
    launch, y = ss.prepare_conv2d(desc, x, wbuf, bias, (2, 2), (3, 3), L.act, sparse=False)
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
        eager = ss.ss_conv2d_dense_fwd(desc, x, wbuf, bias, (2, 2), (3, 3), L.act)
        torch.cuda.synchronize()
        y.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), eager.view(torch.int16)), f"replay {rep}"
