"""The entry point for callers that cannot allocate (ss_conv2d_fwd_static_ws): same result bits as ss_conv2d_fwd, on two
calls in a row that share the library's static scratch array, the second with a smaller input."""
import numpy as np
import pytest
import torch

from paper_2411_00288_amd import workloads as wl
from helpers import dev_bits, host_bits, layer_desc

pytestmark = pytest.mark.gpu


def _L(N, H, W, cin, cout, k, p, dtype, seed):
    return wl.Layer(f"n{N}h{H}w{W}c{cin}o{cout}k{k}", N=N, H=H, W=W, cin=cin, cout=cout, kh=k, kw=k, stride=1, pad=p,
                    dtype=dtype, korder=wl.K_CRS, act=wl.ACT_RELU, mask="logits", seed=seed)


def _both(ss, L):
    d = wl.make_inputs(L)
    desc = layer_desc(ss, L)
    x = dev_bits(d["x"], L.dtype)
    packed = ss.ss_mask_compress(desc, dev_bits(d["W"], L.dtype), torch.from_numpy(d["M"]).cuda())
    bias = torch.from_numpy(d["bias"]).cuda()
    need = ss.ss_conv2d_workspace_bytes(desc, L.N, L.H, L.W, (1, 1), (L.pad,) * 2)
    y_ref = ss.ss_conv2d_fwd(desc, x, packed, bias, (1, 1), (L.pad,) * 2, L.act)
    y = torch.empty_like(y_ref)
    ss.ss_conv2d_fwd_static_ws(desc, x, packed, bias, (1, 1), (L.pad,) * 2, L.act, y=y)
    torch.cuda.synchronize()
    return need, host_bits(y), host_bits(y_ref)


def test_static_workspace_entry_matches_the_workspace_entry_twice_in_a_row(ss):
    ss.ss_debug_force_tile(-1)
    ss.ss_debug_force_split(0)
    # 512 -> 512 3x3 on one 7x7 image: the library splits the reduction by itself (4 tiles, 16 chunks)
    need1, got1, ref1 = _both(ss, _L(1, 7, 7, 512, 512, 3, 1, wl.BF16, 21))
    assert need1 > 0, "the first problem must exercise the scratch array"
    assert np.array_equal(got1, ref1)
    # a smaller input right after it, on the same array: 5x5 image, fewer channels out (two tiles), still split
    need2, got2, ref2 = _both(ss, _L(1, 5, 5, 512, 200, 3, 1, wl.BF16, 22))
    assert 0 < need2 < need1
    assert np.array_equal(got2, ref2)
    # and a problem that needs no scratch at all
    need3, got3, ref3 = _both(ss, _L(2, 9, 9, 64, 96, 3, 1, wl.F16, 23))
    assert need3 == 0
    assert np.array_equal(got3, ref3)


def test_static_workspace_entry_rejects_more_than_the_array_holds(ss):
    L = _L(8, 14, 14, 2048, 512, 1, 0, wl.BF16, 24)      # 1568 pixels x 512 channels, 64 chunks
    d = wl.make_inputs(L)
    desc = layer_desc(ss, L)
    x = dev_bits(d["x"], L.dtype)
    packed = ss.ss_mask_compress(desc, dev_bits(d["W"], L.dtype), torch.from_numpy(d["M"]).cuda())
    ss.ss_debug_force_split(64)
    try:
        assert ss.ss_conv2d_workspace_bytes(desc, L.N, L.H, L.W) > (16 << 20) + (64 << 10)
        with pytest.raises(ss.SSError) as e:
            ss.ss_conv2d_fwd_static_ws(desc, x, packed, None)
        assert e.value.status == ss.SS_ERR_WORKSPACE
    finally:
        ss.ss_debug_force_split(0)
    y = ss.ss_conv2d_fwd_static_ws(desc, x, packed, None)      # unforced: fits (here: no split at all)
    torch.cuda.synchronize()
    assert torch.isfinite(y.float()).all()
