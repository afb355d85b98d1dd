"""Pins for the oracle's weight update V = round16(float(W) + float(U)): the rounding to the storage type is
checked against numpy's float16 and torch's bfloat16 conversions (library routines), on every 16-bit pattern
paired with addends that produce ties, carries, subnormals, cancellation and overflow."""
import numpy as np
import torch

import oracle
from paper_2411_00288_amd import workloads as wl


def _finite(bits, dtype):
    v = oracle.bits_to_double(bits, dtype)
    return np.isfinite(v)


def test_fp16_update_matches_numpy_on_all_patterns():
    allb = np.arange(65536, dtype=np.uint16)
    addends = np.array([0x0000, 0x8000, 0x0001, 0x8001, 0x03FF, 0x0400, 0x1400, 0x3C00, 0xBC00, 0x3C01, 0x3555, 0x7BFF,
                        0xFBFF, 0x4900, 0x0200, 0x6800, 0x2E66, 0xAE66], dtype=np.uint16)
    rng = np.random.default_rng(0)
    addends = np.concatenate([addends, rng.integers(0, 0x7C00, 14).astype(np.uint16)])
    for u in addends:
        U = np.full_like(allb, u)
        keep = _finite(allb, wl.F16)
        got = oracle.update(allb, U, wl.F16)
        with np.errstate(over="ignore", invalid="ignore"):
            ref = (allb.view(np.float16).astype(np.float32) + U.view(np.float16).astype(np.float32)).astype(np.float16)
        assert np.array_equal(got[keep], ref.view(np.uint16)[keep]), hex(int(u))


def test_bf16_update_matches_torch_on_all_patterns():
    allb = np.arange(65536, dtype=np.uint16)
    addends = np.array([0x0000, 0x8000, 0x0001, 0x007F, 0x0080, 0x3F80, 0xBF80, 0x3F81, 0x3EAB, 0x7F7F, 0xFF7F, 0x4300,
                        0x3C00, 0xBC00, 0x3380], dtype=np.uint16)
    rng = np.random.default_rng(1)
    addends = np.concatenate([addends, rng.integers(0, 0x7F80, 15).astype(np.uint16)])
    ta = torch.from_numpy(allb.view(np.int16)).view(torch.bfloat16)
    for u in addends:
        U = np.full_like(allb, u)
        keep = _finite(allb, wl.BF16)
        got = oracle.update(allb, U, wl.BF16)
        tu = torch.from_numpy(U.view(np.int16)).view(torch.bfloat16)
        ref = (ta.float() + tu.float()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(got[keep], ref[keep]), hex(int(u))


def test_update_closed_forms():
    f = lambda *v: wl.to_bits(np.array(v, dtype=np.float32), wl.F16)
    # exact sums, a tie that goes to even (2048 + 1 = 2049 -> 2048; 2050 + 1 = 2051 -> 2052), overflow to infinity
    assert np.array_equal(oracle.update(f(1.0, 2048.0, 2050.0, 65504.0, -1.5), f(2.0, 1.0, 1.0, 65504.0, 1.5), wl.F16),
                          np.array([0x4200, 0x6800, 0x6802, 0x7C00, 0x0000], dtype=np.uint16))
    b = lambda *v: wl.to_bits(np.array(v, dtype=np.float32), wl.BF16)
    # bf16 has 8 significand bits: 256 + 1 -> 256 (tie to even), 258 + 1 -> 260
    assert np.array_equal(oracle.update(b(256.0, 258.0, 1.0), b(1.0, 1.0, 0.5), wl.BF16), b(256.0, 260.0, 1.5))
    # U = 0 leaves every finite pattern untouched (including -0, subnormals)
    allb = np.arange(65536, dtype=np.uint16)
    for dt in (wl.F16, wl.BF16):
        keep = _finite(allb, dt) & (allb != 0x8000)          # (-0) + (+0) = +0
        assert np.array_equal(oracle.update(allb, np.zeros_like(allb), dt)[keep], allb[keep])
