"""Split reduction: several workgroups per output tile, fp32 partial sums and ticket counters in the caller's workspace.

The library splits by itself only where a grid would leave most of the chip idle (few output pixels, long reduction);
the tests also force splits (`ss_debug_force_split`) on every tile shape, and check the workspace contract: the size
query, SS_ERR_WORKSPACE, counters handed back at zero (two calls and HIP-graph replays on one workspace)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2411_00288_amd import workloads as wl
from helpers import check_close, dev_bits, host_bits, layer_desc, oracle_ref, run_gpu

pytestmark = pytest.mark.gpu


def _L(N, H, W, cin, cout, k, s=1, p=0, dtype=wl.F16, act=wl.ACT_RELU, seed=0):
    return wl.Layer(f"n{N}h{H}w{W}c{cin}o{cout}k{k}s{s}d{dtype}", N=N, H=H, W=W, cin=cin, cout=cout, kh=k, kw=k,
                    stride=s, pad=p, dtype=dtype, korder=wl.K_CRS, act=act, mask="logits", seed=seed)


SHAPES = [
    _L(2, 7, 7, 128, 256, 3, p=1),                               # 4 chunks of 32 channels, 98 pixels
    _L(1, 9, 11, 96, 136, 3, s=2, p=1, dtype=wl.BF16, seed=1),   # 3 chunks, stride 2, ragged rows
    _L(2, 5, 5, 512, 160, 1, dtype=wl.BF16, seed=2),             # 1x1, 16 steps = 4 chunks, ragged rows
    _L(3, 6, 7, 416, 72, 1, act=wl.ACT_NONE, seed=3),            # 1x1, 13 steps: 4 chunks, the last one short
]


@pytest.mark.parametrize("nsplit", [2, 3, 4])
@pytest.mark.parametrize("tile", [None, 0, 1, 2, 3, 4, 5])
@pytest.mark.parametrize("L", SHAPES, ids=lambda L: L.name)
def test_split_reduction_matches_oracle(ss, force_tile, force_split, L, tile, nsplit):
    d = wl.make_inputs(L)
    ref = oracle_ref(L, d)
    force_tile(tile)
    force_split(nsplit)
    desc = layer_desc(ss, L)
    assert ss.ss_conv2d_workspace_bytes(desc, L.N, L.H, L.W, (L.stride,) * 2, (L.pad,) * 2) > 0
    check_close(run_gpu(ss, L, d, sparse=True), ref, f"{L.name} sparse tile {tile} split {nsplit}")
    check_close(run_gpu(ss, L, d, sparse=False), ref, f"{L.name} dense tile {tile} split {nsplit}")


@pytest.mark.parametrize("nsplit", [2, 3])
@pytest.mark.parametrize("tile", [1, 4, 5])
def test_split_reduction_is_bit_exact_on_integers(ss, force_tile, force_split, tile, nsplit):
    L = _L(2, 8, 7, 96, 150, 3, p=1, act=wl.ACT_NONE)
    d = wl.make_small_int_inputs(L, seed=tile)
    ref = oracle_ref(L, d)
    assert np.abs(ref).max() <= 2048
    force_tile(tile)
    force_split(nsplit)
    for sparse in (True, False):
        y = run_gpu(ss, L, d, sparse=sparse)
        assert np.array_equal(y.float().cpu().numpy().astype(np.float64), ref)


def _operands(ss, L, d):
    desc = layer_desc(ss, L)
    x = dev_bits(d["x"], L.dtype)
    packed = ss.ss_mask_compress(desc, dev_bits(d["W"], L.dtype), torch.from_numpy(d["M"]).cuda())
    return desc, x, packed, torch.from_numpy(d["bias"]).cuda()


def test_split_with_residual_tail(ss, force_split):
    L = _L(2, 6, 6, 256, 192, 1, dtype=wl.BF16, seed=5)
    d = wl.make_inputs(L)
    rng = np.random.Generator(np.random.PCG64(9))
    res_bits = wl.to_bits(rng.standard_normal((L.N, L.Ho, L.Wo, L.cout), dtype=np.float32), L.dtype)
    ref = oracle.conv2d(d["x"], d["W"], d["M"], cin=L.cin, kh=1, kw=1, korder=L.korder, dtype=L.dtype, bias=d["bias"],
                        act=L.act, residual=res_bits)
    desc, x, packed, bias = _operands(ss, L, d)
    force_split(2)
    y = ss.ss_conv2d_res_fwd(desc, x, packed, bias, dev_bits(res_bits, L.dtype), (1, 1), (0, 0), L.act)
    torch.cuda.synchronize()
    check_close(y, ref, "split + residual")


def test_library_splits_small_grids_by_itself_and_checks_the_workspace(ss):
    # one image, 7x7, 512 -> 512 channels: four 128-row tiles for 256 compute units, 16 chunks
    L = _L(1, 7, 7, 512, 512, 3, p=1, dtype=wl.BF16, seed=6)
    d = wl.make_inputs(L)
    ref = oracle_ref(L, d)
    desc, x, packed, bias = _operands(ss, L, d)
    need = ss.ss_conv2d_workspace_bytes(desc, L.N, L.H, L.W, (1, 1), (1, 1))
    assert need > 0 and need % 256 == 0
    # a large grid needs none
    assert ss.ss_conv2d_workspace_bytes(desc, 64, 14, 14, (1, 1), (1, 1)) == 0
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    y1 = ss.ss_conv2d_fwd(desc, x, packed, bias, (1, 1), (1, 1), L.act, workspace=ws)
    torch.cuda.synchronize()
    check_close(y1, ref, "auto split")
    assert int(ws[:256].view(torch.int32).abs().sum()) == 0, "ticket counters must come back at zero"
    # the same workspace again, without clearing it: the result must be the same bits
    y2 = ss.ss_conv2d_fwd(desc, x, packed, bias, (1, 1), (1, 1), L.act, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(y1), host_bits(y2))
    for bad in (None, torch.zeros(need - 256, dtype=torch.uint8, device="cuda")):
        with pytest.raises(ss.SSError) as e:
            if bad is None:      # the raw call: the convenience wrapper would allocate one
                launch, _ = ss.prepare_conv2d(desc, x, packed, bias, (1, 1), (1, 1), L.act, workspace=torch.zeros(0, dtype=torch.uint8, device="cuda"))
                launch()
            else:
                ss.ss_conv2d_fwd(desc, x, packed, bias, (1, 1), (1, 1), L.act, workspace=bad)
        assert e.value.status == ss.SS_ERR_WORKSPACE


def test_split_under_graph_replay(ss, force_split):
    L = _L(2, 7, 7, 128, 256, 3, p=1, seed=7)
    d = wl.make_inputs(L)
    desc, x, packed, bias = _operands(ss, L, d)
    force_split(4)
    need = ss.ss_conv2d_workspace_bytes(desc, L.N, L.H, L.W, (1, 1), (1, 1))
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    launch, y = ss.prepare_conv2d(desc, x, packed, bias, (1, 1), (1, 1), L.act, workspace=ws)
    launch()
    torch.cuda.synchronize()
    eager = host_bits(y).copy()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        launch()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        launch()
        launch()
    for rep in range(4):
        y.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(host_bits(y), eager), f"replay {rep}"
        x2 = x * 1.0           # the program's own eager work between replays
        torch.cuda.synchronize()
