"""Shared helpers of the GPU parity tests: host<->device marshalling and the acceptance rule."""
import numpy as np
import torch

import oracle
from paper_2411_00288_amd import workloads as wl

REL_L2_TOL = 2e-3          # relative L2 error bound for 16-bit outputs with fp32 accumulation
ELT_TOL = 1e-2             # per element: |err| <= ELT_TOL * (|ref| + 1)


def dev_bits(bits: np.ndarray, dtype: int) -> torch.Tensor:
    tdt = torch.float16 if dtype == wl.F16 else torch.bfloat16
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(tdt)


def host_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def layer_desc(ss, L):
    return ss.make_desc(L.cout, L.cin, L.kh, L.kw, L.dtype, L.korder)


def oracle_ref(L, d, M="layer"):
    return oracle.conv2d(d["x"], d["W"], d["M"] if M == "layer" else M, cin=L.cin, kh=L.kh, kw=L.kw,
                         korder=L.korder, dtype=L.dtype, bias=d["bias"], stride=(L.stride,) * 2,
                         pad=(L.pad,) * 2, act=L.act)


def run_gpu(ss, L, d, sparse=True, bias=True):
    desc = layer_desc(ss, L)
    W = dev_bits(d["W"], L.dtype)
    M = None if d["M"] is None else torch.from_numpy(d["M"]).cuda()
    x = dev_bits(d["x"], L.dtype)
    b = torch.from_numpy(d["bias"]).cuda() if bias else None
    if sparse:
        wbuf = ss.ss_mask_compress(desc, W, M)
        y = ss.ss_conv2d_fwd(desc, x, wbuf, b, (L.stride,) * 2, (L.pad,) * 2, L.act)
    else:
        wbuf = ss.ss_dense_pack(desc, W, M)
        y = ss.ss_conv2d_dense_fwd(desc, x, wbuf, b, (L.stride,) * 2, (L.pad,) * 2, L.act)
    torch.cuda.synchronize()
    return y


def check_close(y_gpu: torch.Tensor, ref: np.ndarray, what=""):
    got = y_gpu.float().cpu().numpy().astype(np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    denom = np.linalg.norm(ref)
    rel = np.linalg.norm(got - ref) / denom if denom > 0 else np.linalg.norm(got - ref)
    slack = np.abs(got - ref) - ELT_TOL * (np.abs(ref) + 1)
    assert rel <= REL_L2_TOL, f"{what}: rel-L2 {rel:.3e} > {REL_L2_TOL}"
    assert slack.max() <= 0, f"{what}: per-element bound exceeded by {slack.max():.3e} at {np.unravel_index(slack.argmax(), ref.shape)}"
    return rel
