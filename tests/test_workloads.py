"""The seeded input generator: determinism, storage rounding, mask recipes, layer tables."""
import numpy as np
import torch

import oracle
from paper_2411_00288_amd import workloads as wl


def test_bf16_and_f16_casts_round_to_nearest_even():
    a = np.random.default_rng(0).standard_normal(20000).astype(np.float32) * 3
    a[:6] = [1.00390625, 1.01171875, -1.00390625, 0.0, 65504.0, 1e-8]   # bf16 ties: to even
    tb = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(wl.to_bits(a, wl.BF16), tb)
    th = torch.from_numpy(a).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(wl.to_bits(a, wl.F16), th)
    assert np.array_equal(wl.from_bits(tb, wl.BF16), torch.from_numpy(a).to(torch.bfloat16).float().numpy())


def test_inputs_are_deterministic_and_masks_valid():
    for L in [wl.CONFIG0, wl.Layer("t", N=1, H=3, W=3, cin=8, cout=5, kh=3, kw=3, pad=1, mask="logits", seed=7,
                                   korder=wl.K_RSC, dtype=wl.BF16)]:
        a, b = wl.make_inputs(L), wl.make_inputs(L)
        for k in a:
            assert np.array_equal(a[k], b[k])
        assert a["W"].shape == a["M"].shape == (L.cout, L.K)
        assert a["x"].shape == (L.N, L.H, L.W, L.cin)
        assert oracle.mask_check(a["M"])[0] == 0
        assert (wl.from_bits(a["x"], L.dtype) >= 0).all()          # ReLU(N(0,1))


def test_top2_mask_keeps_largest_magnitudes_ties_to_lower_position():
    Wb = wl.to_bits(np.array([[1, -3, 2, 0.5, 2, 2, 2, 2, -1, 1, 0, 0]], dtype=np.float32), wl.F16)
    assert wl.mask_top2(Wb, wl.F16).tolist() == [[0, 1, 1, 0, 1, 1, 0, 0, 1, 1, 0, 0]]


def test_config_shapes_and_work_match_the_stated_sizes():
    assert wl.CONFIG0.K == 576 and wl.CONFIG0.dense_equiv_flop == 18_874_368
    assert wl.CONFIG1.K == 2304 and wl.CONFIG1.P == 6272 and wl.CONFIG1.dense_equiv_flop == 7_398_752_256
    assert wl.CONFIG1.algorithmic_bytes(True) == 7_087_104 and wl.CONFIG1.algorithmic_bytes(False) == 7_603_200
    assert wl.CONFIG2.dense_equiv_flop == 6_576_668_672 and wl.CONFIG2.algorithmic_bytes(True) == 32_408_576
    rn = wl.resnet50_layers()
    assert sum(l.count for l in rn) == 53 and sum(l.count for l in rn if l.mask != "none") == 48
    assert abs(sum(l.count * l.dense_equiv_flop for l in rn) / 1e9 - 523.2) < 0.5
    cx = wl.convnext_t_stage1_layers()
    assert abs(sum(l.count * l.dense_equiv_flop for l in cx) / 1e9 - 192.4) < 0.5
    assert all(l.K % 4 == 0 for l in rn + cx if l.mask != "none")
