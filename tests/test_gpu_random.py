"""A seeded random sweep of small layer shapes through every entry point of the convolution, against the oracle:
breadth over geometry (ragged sizes, strides, pads, kernel shapes), operand types, flattenings and tails that the
hand-picked cases may have missed."""
import numpy as np
import pytest
import torch

import oracle
from paper_2411_00288_amd import workloads as wl
from helpers import check_close, dev_bits

pytestmark = pytest.mark.gpu

N_CASES = 72


def _draw(seed):
    rng = np.random.Generator(np.random.PCG64(10_000 + seed))
    dtype = [wl.F16, wl.BF16, wl.I8, wl.F8][seed % 4]
    k = int(rng.choice([1, 1, 2, 3, 3, 5]))
    korder = int(rng.choice([wl.K_CRS, wl.K_RSC]))
    if dtype in (wl.I8, wl.F8):
        cin = int(rng.choice([16, 32, 48, 64, 128]))
        if korder == wl.K_CRS and k > 1 and not (k in (2, 3) and cin % 64 == 0):
            korder = wl.K_RSC
    else:
        cin = int(rng.choice([4, 8, 12, 16, 24, 32, 40, 64, 96]))
    stride = int(rng.choice([1, 1, 2]))
    pad = int(rng.integers(0, k // 2 + 2))
    H = int(rng.integers(max(1, k - 2 * pad), 18))
    W = int(rng.integers(max(1, k - 2 * pad), 18))
    N = int(rng.integers(1, 4))
    cout = int(rng.integers(1, 200))
    act = int(rng.choice([wl.ACT_NONE, wl.ACT_RELU, wl.ACT_GELU]))
    residual = bool(rng.integers(0, 2)) and dtype in (wl.F16, wl.BF16)
    L = wl.Layer(f"rnd{seed}", N=N, H=H, W=W, cin=cin, cout=cout, kh=k, kw=k, stride=stride, pad=pad, dtype=dtype,
                 korder=korder, act=act, mask="logits", relu_input=bool(rng.integers(0, 2)), seed=seed)
    return L, residual


@pytest.mark.parametrize("seed", range(N_CASES))
def test_random_layer_matches_oracle(ss, seed):
    L, with_res = _draw(seed)
    assert L.Ho >= 1 and L.Wo >= 1 and L.K % 4 == 0
    desc = ss.make_desc(L.cout, L.cin, L.kh, L.kw, L.dtype, L.korder)
    st, pd = (L.stride,) * 2, (L.pad,) * 2
    kw = dict(cin=L.cin, kh=L.kh, kw=L.kw, korder=L.korder, stride=st, pad=pd, act=L.act)
    M = None
    if L.dtype in (wl.F16, wl.BF16):
        d = wl.make_inputs(L)
        res_bits = None
        if with_res:
            rng = np.random.Generator(np.random.PCG64(77 + seed))
            res_bits = wl.to_bits(rng.standard_normal((L.N, L.Ho, L.Wo, L.cout), dtype=np.float32), L.dtype)
        ref = oracle.conv2d(d["x"], d["W"], d["M"], dtype=L.dtype, bias=d["bias"], residual=res_bits, **kw)
        W, x = dev_bits(d["W"], L.dtype), dev_bits(d["x"], L.dtype)
        M = torch.from_numpy(d["M"]).cuda()
        b = torch.from_numpy(d["bias"]).cuda()
        if with_res:
            r = dev_bits(res_bits, L.dtype)
            ys = ss.ss_conv2d_res_fwd(desc, x, ss.ss_mask_compress(desc, W, M), b, r, st, pd, L.act)
            yd = ss.ss_conv2d_dense_res_fwd(desc, x, ss.ss_dense_pack(desc, W, M), b, r, st, pd, L.act)
        else:
            ys = ss.ss_conv2d_fwd(desc, x, ss.ss_mask_compress(desc, W, M), b, st, pd, L.act)
            yd = ss.ss_conv2d_dense_fwd(desc, x, ss.ss_dense_pack(desc, W, M), b, st, pd, L.act)
    else:
        d = wl.make_inputs_q8(L) if L.dtype == wl.I8 else wl.make_inputs_f8(L)
        fn = oracle.conv2d_q8 if L.dtype == wl.I8 else oracle.conv2d_f8
        ref = fn(d["x"], d["W"], d["M"], scale=d["scale"], bias=d["bias"], **kw)
        W, x = torch.from_numpy(d["W"]).cuda(), torch.from_numpy(d["x"]).cuda()
        M = torch.from_numpy(d["M"]).cuda()
        sc, b = torch.from_numpy(d["scale"]).cuda(), torch.from_numpy(d["bias"]).cuda()
        ys = ss.ss_conv2d_q8_fwd(desc, x, ss.ss_mask_compress(desc, W, M), sc, b, st, pd, L.act)
        yd = ss.ss_conv2d_q8_dense_fwd(desc, x, ss.ss_dense_pack(desc, W, M), sc, b, st, pd, L.act)
    torch.cuda.synchronize()
    what = f"{L.name}: N{L.N} {L.H}x{L.W} cin{L.cin} cout{L.cout} k{L.kh} s{L.stride} p{L.pad} dt{L.dtype} ko{L.korder} act{L.act} res{with_res}"
    check_close(ys, ref, what + " sparse")
    check_close(yd, ref, what + " dense")
