"""Set-up-time checks at the C ABI: a weight buffer that does not belong to the descriptor is refused before any
asynchronous convolution call multiplies it, and the binding refuses operands shorter than the size queries."""
import numpy as np
import pytest
import torch

from paper_2411_00288_amd import workloads as wl
from helpers import dev_bits, layer_desc

pytestmark = pytest.mark.gpu

L = wl.Layer("chk", N=1, H=6, W=6, cin=32, cout=40, kh=3, kw=3, stride=1, pad=1, dtype=wl.F16, mask="logits", seed=5)


def _status(ss, fn):
    with pytest.raises(ss.SSError) as e:
        fn()
    return e.value.status


def test_weights_check_accepts_matching_buffers_and_refuses_the_rest(ss):
    d = wl.make_inputs(L)
    desc = layer_desc(ss, L)
    W, M = dev_bits(d["W"], L.dtype), torch.from_numpy(d["M"]).cuda()
    packed = ss.ss_mask_compress(desc, W, M)
    dense = ss.ss_dense_pack(desc, W, M)
    ss.ss_weights_check(desc, packed, sparse=True)
    ss.ss_weights_check(desc, dense, sparse=False)
    # a dense operand offered as sparse and the reverse (the dense buffer is the larger one, so sizes pass)
    assert _status(ss, lambda: ss.ss_weights_check(desc, dense, sparse=True)) == ss.SS_ERR_INVALID_ARG
    big = torch.zeros(ss.ss_dense_bytes(desc), dtype=torch.uint8, device="cuda")
    big[:packed.numel()] = packed
    assert _status(ss, lambda: ss.ss_weights_check(desc, big, sparse=False)) == ss.SS_ERR_INVALID_ARG
    # packed for another descriptor: other flattening, other type, other shape with the same byte count
    for other in (ss.make_desc(L.cout, L.cin, L.kh, L.kw, L.dtype, wl.K_RSC),
                  ss.make_desc(L.cout, L.cin, L.kh, L.kw, wl.BF16, L.korder),
                  ss.make_desc(L.cout, L.cin * 9, 1, 1, L.dtype, L.korder)):
        assert ss.ss_packed_bytes(other) == ss.ss_packed_bytes(desc)
        assert _status(ss, lambda: ss.ss_weights_check(other, packed, sparse=True)) == ss.SS_ERR_INVALID_ARG
    # a buffer that never saw a packing call
    assert _status(ss, lambda: ss.ss_weights_check(desc, torch.zeros_like(packed), sparse=True)) == ss.SS_ERR_INVALID_ARG


def test_weights_check_reports_a_rejected_mask(ss):
    d = wl.make_inputs(L)
    desc = layer_desc(ss, L)
    M = d["M"].copy()
    M[3, 8:12] = (1, 1, 1, 0)
    packed = torch.empty(ss.ss_packed_bytes(desc), dtype=torch.uint8, device="cuda")
    assert _status(ss, lambda: ss.ss_mask_compress(desc, dev_bits(d["W"], L.dtype), torch.from_numpy(M).cuda(), packed)) \
        == ss.SS_ERR_BAD_MASK
    assert _status(ss, lambda: ss.ss_weights_check(desc, packed, sparse=True)) == ss.SS_ERR_BAD_MASK


def test_binding_refuses_short_operands(ss):
    d = wl.make_inputs(L)
    desc = layer_desc(ss, L)
    x = dev_bits(d["x"], L.dtype)
    packed = ss.ss_mask_compress(desc, dev_bits(d["W"], L.dtype), torch.from_numpy(d["M"]).cuda())
    bias = torch.from_numpy(d["bias"]).cuda()
    assert _status(ss, lambda: ss.ss_conv2d_fwd(desc, x, packed[:-16], bias, (1, 1), (1, 1))) == ss.SS_ERR_INVALID_ARG
    assert _status(ss, lambda: ss.ss_conv2d_fwd(desc, x, packed, bias[:-1], (1, 1), (1, 1))) == ss.SS_ERR_INVALID_ARG
    # a packed buffer is shorter than the dense form: the twin must refuse it
    assert _status(ss, lambda: ss.ss_conv2d_dense_fwd(desc, x, packed, bias, (1, 1), (1, 1))) == ss.SS_ERR_INVALID_ARG
    y = ss.ss_conv2d_fwd(desc, x, packed, bias, (1, 1), (1, 1))
    torch.cuda.synchronize()
    assert np.isfinite(y.float().cpu().numpy()).all()
