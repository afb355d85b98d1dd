"""GPU parity of the masked convolution (sparse path and dense twin) against the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2411_00288_amd import workloads as wl
from helpers import check_close, dev_bits, host_bits, layer_desc, oracle_ref, run_gpu

pytestmark = pytest.mark.gpu


def L_(N, H, W, cin, cout, k, s=1, p=0, dtype=wl.F16, korder=wl.K_CRS, act=wl.ACT_RELU, mask="logits", seed=0, kw=None):
    return wl.Layer(f"n{N}h{H}w{W}c{cin}o{cout}k{k}s{s}p{p}d{dtype}o{korder}", N=N, H=H, W=W, cin=cin, cout=cout,
                    kh=k, kw=k if kw is None else kw, stride=s, pad=p, dtype=dtype, korder=korder, act=act, mask=mask,
                    seed=seed)


SMALL = [
    # pointwise (vector staging): several tiles in both directions and ragged tails
    L_(2, 9, 7, 64, 64, 1),                           # P = 126 (ragged pixel tile)
    L_(3, 10, 10, 128, 160, 1, dtype=wl.BF16),        # P = 300, Cout = 160 (ragged row tile)
    L_(1, 5, 5, 96, 40, 1, dtype=wl.BF16),            # K = 96: odd number of 32-steps
    L_(1, 3, 3, 8, 4, 1),                             # tiny: one block, K = 8
    L_(2, 8, 8, 32, 70, 1, s=2),                      # strided pointwise
    L_(4, 14, 14, 256, 200, 1, mask="top2"),          # P = 784 -> big tiles
    # channels-last flattening (vector staging with taps)
    L_(2, 9, 7, 32, 48, 3, p=1, korder=wl.K_RSC),
    L_(1, 12, 11, 16, 33, 3, s=2, p=1, korder=wl.K_RSC, dtype=wl.BF16),
    L_(2, 8, 8, 24, 64, 2, s=2, korder=wl.K_RSC),     # 2x2 stride 2, K = 96
    L_(1, 6, 6, 8, 16, 5, p=2, korder=wl.K_RSC),      # cin < chunk
    # the paper's flattening (channel slowest): groups span kernel taps
    L_(2, 9, 7, 32, 48, 3, p=1),
    L_(1, 16, 16, 64, 64, 3, p=1, mask="top2", act=wl.ACT_NONE),
    L_(1, 12, 11, 16, 33, 3, s=2, p=1, dtype=wl.BF16),
    L_(2, 8, 8, 24, 64, 2, s=2),
    L_(1, 7, 7, 4, 8, 3, p=1),                        # K = 36: one ragged step
    L_(1, 6, 5, 12, 16, 1, kw=3, p=0),                # 1x3 kernel
    L_(5, 14, 14, 64, 136, 3, p=1, dtype=wl.BF16),    # P = 980 -> big tiles, ragged both ways
    L_(1, 4, 4, 4, 4, 4, p=0),                        # kernel as large as the image
    L_(1, 3, 3, 4, 4, 3, p=2),                        # padding larger than usual
]


@pytest.mark.parametrize("L", SMALL, ids=lambda L: L.name)
def test_sparse_conv_matches_oracle(ss, L):
    d = wl.make_inputs(L)
    y = run_gpu(ss, L, d, sparse=True)
    check_close(y, oracle_ref(L, d), L.name)


@pytest.mark.parametrize("L", SMALL, ids=lambda L: L.name)
def test_dense_twin_matches_oracle(ss, L):
    d = wl.make_inputs(L)
    y = run_gpu(ss, L, d, sparse=False)
    check_close(y, oracle_ref(L, d), L.name)


EXACT = [
    L_(2, 7, 6, 32, 40, 3, p=1), L_(2, 7, 6, 32, 40, 3, p=1, korder=wl.K_RSC), L_(3, 9, 9, 64, 72, 1),
    L_(1, 9, 8, 16, 24, 3, s=2, p=1, dtype=wl.BF16), L_(1, 8, 8, 8, 36, 2, s=2, dtype=wl.BF16, korder=wl.K_RSC),
    L_(4, 14, 14, 32, 130, 3, p=1, act=wl.ACT_NONE),
]


@pytest.mark.parametrize("sparse", [True, False])
@pytest.mark.parametrize("L", EXACT, ids=lambda L: L.name)
def test_small_integer_inputs_are_bit_exact(ss, L, sparse):
    # w in {-1,0,1}, x in {0,1,2}, integer bias: |sum| <= 2*K/2 + 2 stays inside the exact-integer
    # range of the storage type (2048 for fp16, 256 for bf16), so nothing is ever rounded.
    assert L.K + 2 <= (2048 if L.dtype == wl.F16 else 256)
    d = wl.make_small_int_inputs(L, seed=5)
    y = run_gpu(ss, L, d, sparse=sparse)
    ref = oracle_ref(L, d)
    assert np.array_equal(y.float().cpu().numpy().astype(np.float64), ref)
    assert np.array_equal(host_bits(y), wl.to_bits(ref.astype(np.float32), L.dtype))


def test_no_bias_and_no_activation(ss):
    L = L_(2, 6, 6, 32, 32, 3, p=1, act=wl.ACT_NONE)
    d = wl.make_inputs(L)
    y = run_gpu(ss, L, d, sparse=True, bias=False)
    d2 = dict(d, bias=np.zeros_like(d["bias"]))
    check_close(y, oracle_ref(L, d2))


def test_sparse_and_twin_agree_closely(ss):
    # same products in a different order: the two GPU paths differ by fp32 summation order only
    L = L_(2, 14, 14, 128, 128, 3, p=1)
    d = wl.make_inputs(L)
    ys, yd = run_gpu(ss, L, d, True), run_gpu(ss, L, d, False)
    diff = (ys.float() - yd.float()).abs().max().item()
    assert diff <= 2 ** -8 * max(1.0, ys.float().abs().max().item())


def test_config0_full(ss):
    L = wl.CONFIG0
    d = wl.make_inputs(L)
    ref = oracle_ref(L, d)
    check_close(run_gpu(ss, L, d, True), ref, "cfg0 sparse")
    check_close(run_gpu(ss, L, d, False), ref, "cfg0 dense")


def test_config1_full(ss):
    L = wl.CONFIG1
    d = wl.make_inputs(L)
    ref = oracle_ref(L, d)
    r = check_close(run_gpu(ss, L, d, True), ref, "cfg1 sparse")
    check_close(run_gpu(ss, L, d, False), ref, "cfg1 dense")
    assert r < 5e-4          # fp16 output rounding alone is about 2e-4


def test_config2_full(ss):
    L = wl.CONFIG2
    d = wl.make_inputs(L)
    ref = oracle_ref(L, d)
    check_close(run_gpu(ss, L, d, True), ref, "cfg2 sparse")
    check_close(run_gpu(ss, L, d, False), ref, "cfg2 dense")


def test_dense_only_layers_k_not_multiple_of_4(ss):
    # the ResNet stem shape class: cin = 3, 7x7, stride 2 (stays dense; the sparse call rejects it)
    L = L_(2, 20, 20, 3, 16, 7, s=2, p=3, dtype=wl.BF16, mask="none")
    d = wl.make_inputs(L)
    check_close(run_gpu(ss, L, d, sparse=False), oracle_ref(L, d))
    with pytest.raises(ss.SSError) as ei:
        ss.ss_packed_bytes(layer_desc(ss, L))
    assert ei.value.status == ss.SS_ERR_UNSUPPORTED


def test_argument_errors(ss):
    L = L_(1, 4, 4, 8, 8, 3, p=1)
    d = wl.make_inputs(L)
    desc = layer_desc(ss, L)
    x = dev_bits(d["x"], L.dtype)
    packed = ss.ss_mask_compress(desc, dev_bits(d["W"], L.dtype), torch.from_numpy(d["M"]).cuda())
    with pytest.raises(ss.SSError):                    # unknown activation
        ss.ss_conv2d_fwd(desc, x, packed, None, (1, 1), (1, 1), 7)
    with pytest.raises(ss.SSError):                    # zero stride
        ss.ss_conv2d_fwd(desc, x, packed, None, (0, 1), (1, 1), 0)
    with pytest.raises(ss.SSError):                    # kernel larger than padded input
        ss.ss_conv2d_fwd(ss.make_desc(8, 8, 7, 7), x, packed, None, (1, 1), (0, 0), 0)
    with pytest.raises(ss.SSError):                    # wrong channel count
        ss.ss_conv2d_fwd(ss.make_desc(8, 16, 3, 3), x, packed, None, (1, 1), (1, 1), 0)
    with pytest.raises(ss.SSError):                    # host tensor
        ss.ss_conv2d_fwd(desc, x.cpu(), packed, None, (1, 1), (1, 1), 0)


def test_prepared_launch_in_hip_graph_replays_correctly(ss):
    # The benchmark records launches in a HIP graph.  Replay several times with eager work and
    # synchronisation in between, on changing input contents, and compare with the eager result.
    L = L_(2, 14, 14, 64, 96, 3, p=1)
    d = wl.make_inputs(L)
    desc = layer_desc(ss, L)
    x = dev_bits(d["x"], L.dtype)
    packed = ss.ss_mask_compress(desc, dev_bits(d["W"], L.dtype), torch.from_numpy(d["M"]).cuda())
    bias = torch.from_numpy(d["bias"]).cuda()
    launch, y = ss.prepare_conv2d(desc, x, packed, bias, (1, 1), (1, 1), L.act)
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
        eager = ss.ss_conv2d_fwd(desc, x, packed, bias, (1, 1), (1, 1), L.act)
        torch.cuda.synchronize()
        y.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y.view(torch.int16), eager.view(torch.int16)), f"replay {rep}"
