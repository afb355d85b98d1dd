"""Full-size layers of the ResNet-50 (batch 64) and ConvNeXt-T stage-1 (batch 128) workloads, in the
launch configuration the benchmark times, checked on sampled outputs that the oracle computes one by
one (the full tensors would take the CPU minutes)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2411_00288_amd import workloads as wl
from helpers import ELT_TOL, REL_L2_TOL, run_gpu

pytestmark = pytest.mark.gpu

NPTS = 4096


def _pick(layers, names):
    by = {l.name: l for l in layers}
    return [by[n] for n in names]


LAYERS = (_pick(wl.resnet50_layers(), ["stem_7x7_3_64_s2", "s1_c3_1x1_64_256", "s1_c2_3x3_64_64", "s2_c2_3x3_128_128_s2",
                                        "s3_c2_3x3_256_256", "s4_c2_3x3_512_512", "s4_c1_1x1_2048_512", "s3_ds_1x1_512_1024_s2"])
          + wl.convnext_t_stage1_layers())


@pytest.mark.parametrize("L", LAYERS, ids=lambda L: L.name)
def test_full_size_layer_on_sampled_outputs(ss, L):
    d = wl.make_inputs(L)
    sparse = L.mask != "none"
    y = run_gpu(ss, L, d, sparse=sparse)
    total = L.P * L.cout
    rng = np.random.default_rng(L.seed)
    idx = np.unique(np.concatenate([rng.integers(0, total, size=NPTS),
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
