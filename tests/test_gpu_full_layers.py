"""Every unique layer shape of the ResNet-50 (batch 64) and ConvNeXt-T stage-1 (batch 128) workloads at full size,
in the launch configuration the benchmark times, checked on sampled outputs that the oracle computes one by one
(the full tensors would take the CPU minutes).  The sample is stratified: at least one output from every 64-channel
x 64-pixel block of the output matrix, which is the granularity of the smallest workgroup tile, so every workgroup
of whichever tile the library picks contributes a checked element; plus a uniform random draw and the first and
last pixels."""
import numpy as np
import pytest
import torch

import oracle
from paper_2411_00288_amd import workloads as wl
from helpers import ELT_TOL, REL_L2_TOL, run_gpu

pytestmark = pytest.mark.gpu

NPTS = 4096


LAYERS = (wl.resnet50_layers() + wl.convnext_t_stage1_layers()      # the 24 + 3 unique shapes (depthwise is not in the list)
          # the headline layer at the two scaled batch sizes the benchmark reports (the resident-grid kernel's launches)
          + [wl.with_batch(wl.CONFIG1, 500), wl.with_batch(wl.CONFIG1, 512)])


def stratified_indices(L, rng, block=64):
    """Flat indices (pixel * cout + channel) with one uniformly drawn element per block x block tile of [P][cout]."""
    nb_p, nb_o = -(-L.P // block), -(-L.cout // block)
    bp, bo = np.meshgrid(np.arange(nb_p, dtype=np.int64), np.arange(nb_o, dtype=np.int64), indexing="ij")
    pp = np.minimum(bp * block + rng.integers(0, block, size=bp.shape), L.P - 1)
    oo = np.minimum(bo * block + rng.integers(0, block, size=bo.shape), L.cout - 1)
    return (pp * L.cout + oo).reshape(-1)


@pytest.mark.parametrize("L", LAYERS, ids=lambda L: L.name)
def test_full_size_layer_on_sampled_outputs(ss, L):
    d = wl.make_inputs(L)
    sparse = L.mask != "none"
    y = run_gpu(ss, L, d, sparse=sparse)
    total = L.P * L.cout
    rng = np.random.default_rng(L.seed)
    idx = np.unique(np.concatenate([rng.integers(0, total, size=NPTS), stratified_indices(L, rng),
                                    np.arange(0, min(total, 64)),                  # first pixel's channels
                                    np.arange(total - 64, total)]))                # last pixel's channels
    ref = oracle.conv2d_points(d["x"], d["W"], d["M"], idx, cin=L.cin, kh=L.kh, kw=L.kw, korder=L.korder, dtype=L.dtype,
                               bias=d["bias"], stride=(L.stride,) * 2, pad=(L.pad,) * 2, act=L.act)
    got = y.reshape(-1)[torch.from_numpy(idx).cuda()].float().cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)
    assert rel <= REL_L2_TOL, f"{L.name}: rel-L2 {rel:.3e}"
    assert (np.abs(got - ref) <= ELT_TOL * (np.abs(ref) + 1)).all()
    if sparse:   # the twin sees the same inputs
        yd = run_gpu(ss, L, d, sparse=False)
        gd = yd.reshape(-1)[torch.from_numpy(idx).cuda()].float().cpu().numpy().astype(np.float64)
        assert np.linalg.norm(gd - ref) / max(np.linalg.norm(ref), 1e-30) <= REL_L2_TOL
        assert (np.abs(gd - ref) <= ELT_TOL * (np.abs(ref) + 1)).all()
