"""The chained ResNet-50 convolution trunk (stem -> max pool -> 16 bottlenecks with fused add + ReLU tails) on a small
image: every op is checked against the oracle on the inputs the GPU actually fed it (so a wrong buffer, a missing
residual or a wrong stride shows up at the op where it happens), the pooling bit for bit, and the final feature map
against an oracle-only chain."""
import numpy as np
import pytest
import torch

import oracle
from helpers import check_close, host_bits
from paper_2411_00288_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _conv_ref(L, d, x_bits, res_bits):
    return oracle.conv2d(x_bits, d["W"], d["M"], cin=L.cin, kh=L.kh, kw=L.kw, korder=L.korder, dtype=L.dtype,
                         bias=d["bias"], stride=(L.stride,) * 2, pad=(L.pad,) * 2, act=L.act, residual=res_bits)


@pytest.mark.parametrize("sparse,channels", [(True, 4), (False, 4), (True, 3)])
def test_trunk_ops_match_oracle_on_their_actual_inputs(ss, sparse, channels):
    from paper_2411_00288_amd import resnet50
    t = resnet50.Trunk(batch=1, image=64, dtype=wl.BF16, sparse=sparse, keep_host=True, image_channels=channels,
                       fuse_pairs=False)                        # every layer writes its own buffer
    assert sum(op.kind == "conv" for op in t.ops) == 53 and t.output.shape == (1, 2, 2, 2048)
    rng = np.random.Generator(np.random.PCG64(77))
    x = rng.standard_normal((1, 64, 64, channels), dtype=np.float32)
    x[..., 3:] = 0                                              # the padding channel of the image
    x_bits = wl.to_bits(x, wl.BF16)
    t.input.copy_(torch.from_numpy(x_bits.view(np.int16)).cuda().view(torch.bfloat16))
    t.forward()
    torch.cuda.synchronize()
    got = {i: host_bits(b) for i, b in t.bufs.items()}
    chain = {0: x_bits}                                         # oracle-only chain, rounded to bf16 after every op
    for op in t.ops:
        if op.kind == "pool":
            assert np.array_equal(got[op.dst], oracle.maxpool2d(got[op.src], dtype=wl.BF16, k=3, stride=2, pad=1)), op.name
            chain[op.dst] = oracle.maxpool2d(chain[op.src], dtype=wl.BF16, k=3, stride=2, pad=1)
            continue
        L, d = op.layer, t.host[op.name]
        res = None if op.residual is None else got[op.residual]
        check_close(t.bufs[op.dst], _conv_ref(L, d, got[op.src], res), op.name)
        cres = None if op.residual is None else chain[op.residual]
        chain[op.dst] = wl.to_bits(_conv_ref(L, d, chain[op.src], cres).astype(np.float32), wl.BF16)
    # end to end: rounding decisions differ between fp32 and fp64 accumulation and propagate through 50 layers
    final = oracle.bits_to_double(chain[t.ops[-1].dst], wl.BF16)
    out = t.output.float().cpu().numpy().astype(np.float64)
    assert np.isfinite(out).all()
    assert np.linalg.norm(out - final) / np.linalg.norm(final) <= 3e-2


def test_trunk_replays_in_a_hip_graph(ss):
    from paper_2411_00288_amd import resnet50
    t = resnet50.Trunk(batch=2, image=64, dtype=wl.BF16, sparse=True)
    t.input.copy_(torch.randn(t.input.shape, device="cuda").to(torch.bfloat16))
    t.forward()
    torch.cuda.synchronize()
    eager = t.output.clone()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            t.forward()
    for _ in range(3):
        t.output.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(t.output.view(torch.int16), eager.view(torch.int16))


def test_maxpool_matches_oracle_bit_for_bit(ss):
    rng = np.random.Generator(np.random.PCG64(5))
    for dtype, shape, k, s, p in [(wl.BF16, (2, 17, 13, 64), 3, 2, 1), (wl.F16, (1, 8, 8, 8), 2, 2, 0), (wl.F16, (3, 9, 9, 24), 3, 1, 1)]:
        xb = wl.to_bits(rng.standard_normal(shape, dtype=np.float32), dtype)
        tdt = torch.float16 if dtype == wl.F16 else torch.bfloat16
        y = ss.ss_maxpool2d(torch.from_numpy(xb.view(np.int16)).cuda().view(tdt), k, s, p)
        assert np.array_equal(host_bits(y), oracle.maxpool2d(xb, dtype=dtype, k=k, stride=s, pad=p))
    with pytest.raises(ss.SSError):
        ss.ss_maxpool2d(torch.zeros((1, 4, 4, 12), dtype=torch.float16, device="cuda"))       # C % 8 != 0


@pytest.mark.parametrize("sparse", [True, False])
def test_trunk_with_fused_pairs_equals_the_unfused_trunk(ss, sparse):
    """Running a block's 3x3 and 1x1 expansion as one kernel changes only the order of fp32 additions in the 1x1."""
    from paper_2411_00288_amd import resnet50
    a = resnet50.Trunk(batch=2, image=64, dtype=wl.BF16, sparse=sparse, fuse_pairs=False)
    b = resnet50.Trunk(batch=2, image=64, dtype=wl.BF16, sparse=sparse, fuse_pairs=True)
    assert len(b.fused) == (7 if sparse else 3) and len(b.launches) == len(a.launches) - len(b.fused)
    x = torch.randn(a.input.shape, device="cuda").to(torch.bfloat16)
    x[..., 3:] = 0
    a.input.copy_(x)
    b.input.copy_(x)
    a.forward()
    b.forward()
    torch.cuda.synchronize()
    ya, yb = a.output.float(), b.output.float()
    assert torch.isfinite(yb).all()
    assert (torch.linalg.norm(ya - yb) / torch.linalg.norm(ya)).item() <= 1e-2
    # the buffers of the stages that do not fuse anything upstream are identical
    first_c1 = next(op for op in a.ops if op.name == "s1b0_c1")
    assert torch.equal(a.bufs[first_c1.dst], b.bufs[first_c1.dst])
