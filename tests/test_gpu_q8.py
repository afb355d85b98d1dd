"""GPU parity of the 8-bit integer precision point, through the C ABI: packing bit for bit, the convolution against
the oracle's exact integer sums (bit for bit where the 16-bit output can hold them, else to half an output ulp)."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from oracle import device_layout as dl
from paper_2411_00288_amd import workloads as wl

pytestmark = pytest.mark.gpu

TILE_IDS = [0, 1, 2, 3, 4, 5]


def _L(N, H, W, cin, cout, k, s=1, p=0, korder=wl.K_RSC, act=wl.ACT_RELU, seed=0, mask="logits"):
    return wl.Layer(f"q8n{N}h{H}w{W}c{cin}o{cout}k{k}s{s}", N=N, H=H, W=W, cin=cin, cout=cout, kh=k, kw=k, stride=s, pad=p,
                    dtype=wl.I8, korder=korder, act=act, mask=mask, seed=seed)


def _desc(ss, L):
    return ss.make_desc(L.cout, L.cin, L.kh, L.kw, wl.I8, L.korder)


def _run(ss, L, d, sparse=True, scale=True, bias=True, act=None):
    desc = _desc(ss, L)
    W = torch.from_numpy(d["W"]).cuda()
    M = None if d["M"] is None else torch.from_numpy(d["M"]).cuda()
    x = torch.from_numpy(d["x"]).cuda()
    sc = torch.from_numpy(d["scale"]).cuda() if scale else None
    b = torch.from_numpy(d["bias"]).cuda() if bias else None
    act = L.act if act is None else act
    if sparse:
        y = ss.ss_conv2d_q8_fwd(desc, x, ss.ss_mask_compress(desc, W, M), sc, b, (L.stride,) * 2, (L.pad,) * 2, act)
    else:
        y = ss.ss_conv2d_q8_dense_fwd(desc, x, ss.ss_dense_pack(desc, W, M), sc, b, (L.stride,) * 2, (L.pad,) * 2, act)
    torch.cuda.synchronize()
    return y


def _ref(L, d, scale=True, bias=True, act=None):
    return oracle.conv2d_q8(d["x"], d["W"], d["M"], cin=L.cin, kh=L.kh, kw=L.kw, korder=L.korder,
                            scale=d["scale"] if scale else None, bias=d["bias"] if bias else None,
                            stride=(L.stride,) * 2, pad=(L.pad,) * 2, act=L.act if act is None else act)


def check_q8(y, ref, what=""):
    """The integer sum is exact on both sides; what remains is the fp32 evaluation of scale*sum + bias (a few 2^-24
    relative to the terms), the activation, and one rounding to binary16 (half an ulp: 2^-11 relative, 2^-25 absolute
    in the subnormal range).  The bound leaves a few percent of slack over that and 2e-6 for cancellation between
    scale*sum and the bias and for the normal-CDF approximation."""
    got = y.float().cpu().numpy().astype(np.float64)
    assert got.shape == ref.shape and np.isfinite(got).all(), what
    slack = np.abs(got - ref) - (5.2e-4 * np.abs(ref) + 2e-6)
    assert slack.max() <= 0, f"{what}: bound exceeded by {slack.max():.3e} at {np.unravel_index(slack.argmax(), ref.shape)}"


PACK_SHAPES = [  # cout, cin, kh, kw, korder
    (64, 64, 3, 3, wl.K_RSC),      # K = 576 = 9 steps
    (256, 64, 1, 1, wl.K_CRS),
    (40, 8, 3, 3, wl.K_CRS),       # ragged rows, K = 72 (ragged step)
    (7, 4, 1, 1, wl.K_CRS),        # a single block per row
    (96, 24, 2, 2, wl.K_RSC),      # K = 96
    (33, 96, 1, 1, wl.K_CRS),
    (130, 36, 3, 3, wl.K_RSC),     # K = 324
    (1, 4, 1, 1, wl.K_CRS),
]


@pytest.mark.parametrize("shape", PACK_SHAPES)
@pytest.mark.parametrize("mask", ["logits", "top2"])
def test_packed_bytes_match_oracle_bit_for_bit(ss, shape, mask):
    cout, cin, kh, kw, korder = shape
    L = wl.Layer("t", N=1, H=4, W=4, cin=cin, cout=cout, kh=kh, kw=kw, dtype=wl.I8, korder=korder, mask=mask, seed=31)
    d = wl.make_inputs_q8(L)
    Wq = d["W"].copy()
    n = min(4, Wq.size)
    Wq.reshape(-1)[:n] = np.array([-128, 127, 0, -1], dtype=np.int8)[:n]
    desc = _desc(ss, L)
    assert ss.ss_packed_bytes(desc) == dl.packed_bytes8(cout, L.K)
    assert ss.ss_dense_bytes(desc) == dl.dense_bytes8(cout, L.K)
    W, M = torch.from_numpy(Wq).cuda(), torch.from_numpy(d["M"]).cuda()
    W0, M0 = W.clone(), M.clone()
    packed = ss.ss_mask_compress(desc, W, M)
    vals, meta = oracle.compress8(Wq, d["M"])
    got = packed.cpu().numpy()
    assert np.array_equal(got, dl.tile8(vals, meta, cin=cin, kh=kh, kw=kw, korder=korder))
    h, v2, m2 = dl.untile8(got)
    assert np.array_equal(v2, vals) and np.array_equal(m2, meta)
    assert torch.equal(W, W0) and torch.equal(M, M0)                # inputs are never written
    back = ss.ss_mask_decompress(desc, packed).cpu().numpy()
    assert back.dtype == np.int8
    assert np.array_equal(back, np.where(d["M"] == 1, Wq, 0)) and np.array_equal(back, oracle.decompress8(vals, meta))
    Wm = np.where(d["M"] == 1, Wq, 0).astype(np.int8)
    assert np.array_equal(ss.ss_dense_pack(desc, W, M).cpu().numpy(), dl.tile_dense8(Wm, cin=cin, kh=kh, kw=kw, korder=korder))
    assert np.array_equal(ss.ss_dense_pack(desc, W, None).cpu().numpy(), dl.tile_dense8(Wq, cin=cin, kh=kh, kw=kw, korder=korder))


def test_compress_reports_first_invalid_block_and_rejects_updates(ss):
    L = wl.Layer("t", N=1, H=2, W=2, cin=16, cout=70, kh=3, kw=3, dtype=wl.I8, korder=wl.K_RSC, mask="logits", seed=1)
    d = wl.make_inputs_q8(L)
    desc = _desc(ss, L)
    W = torch.from_numpy(d["W"]).cuda()
    Mb = d["M"].copy()
    Mb[41, 20:24] = 1
    Mb[50, 0:4] = 0
    with pytest.raises(ss.SSError) as e:
        ss.ss_mask_compress(desc, W, torch.from_numpy(Mb).cuda())
    assert e.value.status == ss.SS_ERR_BAD_MASK and e.value.detail == (41, 5)
    with pytest.raises(ss.SSError) as e:
        ss.ss_mask_update_compress(desc, W, W.clone(), torch.from_numpy(d["M"]).cuda())
    assert e.value.status in (ss.SS_ERR_UNSUPPORTED, ss.SS_ERR_INVALID_ARG)


SHAPES = [
    _L(3, 14, 14, 64, 300, 3, p=1),                 # 3x3, K = 576 bytes = 9 steps (ragged last chunk of 2), ragged rows / pixels
    _L(2, 13, 11, 128, 200, 3, p=1, korder=wl.K_CRS, seed=6),   # the paper's flattening: byte transpose of the taps, 2 chunks of 64 channels
    _L(2, 12, 12, 64, 136, 2, s=2, korder=wl.K_CRS, seed=7),    # 2x2 stride 2 in the paper's flattening
    _L(2, 9, 10, 128, 200, 3, p=1, seed=4),         # K = 1152 bytes: the long-reduction staging (chunks of 512 bytes), 2.25 chunks
    _L(2, 15, 13, 96, 136, 3, s=2, p=1),            # stride 2
    _L(3, 9, 11, 160, 264, 1, korder=wl.K_CRS),     # pointwise, K = 160 (2.5 steps)
    _L(2, 10, 10, 64, 130, 1),                      # pointwise, a single step (short-reduction staging)
    _L(2, 12, 12, 96, 200, 2, s=2),                 # 2x2 stride 2
    _L(2, 9, 9, 16, 140, 3, p=1),                   # smallest channel count: K = 144
    _L(1, 7, 7, 512, 520, 3, p=1, seed=5),          # long reduction: 72 steps
    _L(2, 11, 12, 48, 64, 5, p=2, seed=2),          # 5x5, cout = 64 (the 64-wide tiles' own path)
]


@pytest.mark.parametrize("L", SHAPES, ids=lambda L: L.name)
def test_convolution_matches_oracle(ss, L):
    d = wl.make_inputs_q8(L)
    ref = _ref(L, d)
    check_q8(_run(ss, L, d, sparse=True), ref, f"{L.name} sparse")
    check_q8(_run(ss, L, d, sparse=False), ref, f"{L.name} dense")


@pytest.mark.parametrize("tile", TILE_IDS)
@pytest.mark.parametrize("L", SHAPES[:8], ids=lambda L: L.name)
def test_every_tile_shape_matches_oracle(ss, force_tile, L, tile):
    d = wl.make_inputs_q8(L)
    ref = _ref(L, d)
    force_tile(tile)
    check_q8(_run(ss, L, d, sparse=True), ref, f"{L.name} sparse tile {tile}")
    check_q8(_run(ss, L, d, sparse=False), ref, f"{L.name} dense tile {tile}")


@pytest.mark.parametrize("tile", TILE_IDS)
def test_integer_sums_are_bit_exact(ss, force_tile, tile):
    """Without scale, bias and activation the output is the integer sum itself; with operands small enough that
    |sum| <= 2048 binary16 holds it exactly, so the GPU must equal the oracle bit for bit."""
    L = _L(3, 10, 9, 64, 150, 3, p=1, act=wl.ACT_NONE)
    rng = np.random.Generator(np.random.PCG64(tile))
    d = {"W": rng.integers(-1, 2, size=(L.cout, L.K)).astype(np.int8),
         "x": rng.integers(-3, 4, size=(L.N, L.H, L.W, L.cin)).astype(np.int8),
         "M": wl.mask_from_logits(rng.standard_normal((L.cout, L.K // 4, 6), dtype=np.float32)),
         "scale": None, "bias": None}
    assert 3 * L.K // 2 <= 2048
    ref = _ref(L, d, scale=False, bias=False)
    force_tile(tile)
    for sparse in (True, False):
        y = _run(ss, L, d, sparse=sparse, scale=False, bias=False)
        assert np.array_equal(y.float().cpu().numpy().astype(np.float64), ref)


def test_extreme_operands_do_not_wrap(ss):
    """-128 x -128 over the whole reduction: the int32 sum (16384 per kept product) stays exact; the scale brings it
    into the output's range."""
    L = _L(1, 6, 6, 128, 64, 3, p=1, act=wl.ACT_NONE, mask="top2")
    d = wl.make_inputs_q8(L)
    d["W"][:] = -128
    d["x"][:] = -128
    d["M"] = np.tile(np.array([1, 0, 0, 1], dtype=np.uint8), (L.cout, L.K // 4))
    d["scale"] = np.full(L.cout, 2.0 ** -14, dtype=np.float32)
    ref = _ref(L, d)
    assert ref.max() > 500          # 16384 * K/2 kept products * 2^-14
    check_q8(_run(ss, L, d, sparse=True), ref, "extreme sparse")
    check_q8(_run(ss, L, d, sparse=False), ref, "extreme dense")


@pytest.mark.parametrize("act", [wl.ACT_NONE, wl.ACT_RELU, wl.ACT_GELU])
def test_layer_tail_variants(ss, act):
    L = _L(2, 9, 9, 64, 96, 3, p=1, seed=7)
    d = wl.make_inputs_q8(L)
    for scale, bias in ((True, True), (True, False), (False, False)):
        dd = dict(d)
        if not scale:      # without a scale the sums themselves (up to ~1e5) must fit binary16: shrink the operands
            dd["W"] = (d["W"] // 32).astype(np.int8)
            dd["x"] = (d["x"] // 16).astype(np.int8)
        ref = _ref(L, dd, scale=scale, bias=bias, act=act)
        assert np.abs(ref).max() < 60000
        check_q8(_run(ss, L, dd, sparse=True, scale=scale, bias=bias, act=act), ref, f"act {act} scale {scale} bias {bias}")


def test_full_size_layer_at_sampled_points(ss):
    """The benchmark's 8-bit layer (the 3x3 256->256 14x14 layer at batch 32, channels-last flattening) in the launch
    configuration the benchmark times, at 4096 sampled outputs."""
    L = wl.Layer("cfg1_q8", N=32, H=14, W=14, cin=256, cout=256, kh=3, kw=3, stride=1, pad=1, dtype=wl.I8,
                 korder=wl.K_RSC, act=wl.ACT_RELU, mask="logits", seed=0)
    d = wl.make_inputs_q8(L)
    idx = np.random.default_rng(1).choice(L.P * L.cout, size=4096, replace=False)
    ref = oracle.conv2d_q8_points(d["x"], d["W"], d["M"], idx, cin=L.cin, kh=3, kw=3, korder=L.korder, scale=d["scale"],
                                  bias=d["bias"], stride=(1, 1), pad=(1, 1), act=L.act)
    for sparse in (True, False):
        y = _run(ss, L, d, sparse=sparse).float().cpu().numpy().astype(np.float64).reshape(-1)[idx]
        assert (np.abs(y - ref) <= 5.2e-4 * np.abs(ref) + 2e-6).all()
    assert (ref > 0).mean() > 0.2


def test_argument_errors(ss):
    L = _L(1, 8, 8, 64, 64, 3, p=1)
    d = wl.make_inputs_q8(L)
    x = torch.from_numpy(d["x"]).cuda()
    W, M = torch.from_numpy(d["W"]).cuda(), torch.from_numpy(d["M"]).cuda()
    desc = _desc(ss, L)
    packed = ss.ss_mask_compress(desc, W, M)

    def status(fn):
        with pytest.raises(ss.SSError) as e:
            fn()
        return e.value.status

    # channel-slowest flattening with taps other than 3x3 / 2x2, or with cin % 64 != 0; channel counts that are not a
    # multiple of 16
    crs5 = ss.make_desc(L.cout, L.cin, 5, 5, wl.I8, wl.K_CRS)
    p5 = torch.zeros(ss.ss_packed_bytes(crs5), dtype=torch.uint8, device="cuda")
    assert status(lambda: ss.ss_conv2d_q8_fwd(crs5, x, p5, pad=(2, 2))) == ss.SS_ERR_UNSUPPORTED
    crs48 = ss.make_desc(64, 48, 3, 3, wl.I8, wl.K_CRS)
    x48 = torch.zeros((1, 8, 8, 48), dtype=torch.int8, device="cuda")
    p48 = torch.zeros(ss.ss_packed_bytes(crs48), dtype=torch.uint8, device="cuda")
    assert status(lambda: ss.ss_conv2d_q8_fwd(crs48, x48, p48, pad=(1, 1))) == ss.SS_ERR_UNSUPPORTED
    d8 = ss.make_desc(64, 8, 1, 1, wl.I8, wl.K_CRS)
    x8 = torch.zeros((1, 4, 4, 8), dtype=torch.int8, device="cuda")
    p8 = torch.zeros(ss.ss_packed_bytes(d8), dtype=torch.uint8, device="cuda")
    assert status(lambda: ss.ss_conv2d_q8_fwd(d8, x8, p8)) == ss.SS_ERR_UNSUPPORTED
    # a 16-bit descriptor at the 8-bit entry point, and an 8-bit descriptor at a 16-bit one
    f16 = ss.make_desc(L.cout, L.cin, 3, 3, wl.F16, wl.K_RSC)
    lib = ss.binding._lib
    y = torch.empty((1, 8, 8, 64), dtype=torch.float16, device="cuda")
    vp = lambda t: ctypes.c_void_p(t.data_ptr())
    raw = lambda dsc, out_dtype: lib.ss_conv2d_q8_fwd(ctypes.byref(dsc), vp(x), 1, 8, 8, vp(packed), None, None, 1, 1, 1, 1,
                                                      0, out_dtype, vp(y), None, 0, None)
    assert raw(f16, ss.SS_F16) == ss.SS_ERR_INVALID_ARG
    assert raw(desc, ss.SS_BF16) == ss.SS_ERR_UNSUPPORTED
    assert raw(desc, 7) == ss.SS_ERR_INVALID_ARG
    assert raw(desc, ss.SS_F16) == ss.SS_OK
    xh = torch.zeros((1, 8, 8, 64), dtype=torch.float16, device="cuda")
    st = lib.ss_conv2d_fwd(ctypes.byref(desc), vp(xh), 1, 8, 8, vp(packed), None, 1, 1, 1, 1, 0, vp(y), None, 0, None)
    assert st == ss.SS_ERR_UNSUPPORTED
    torch.cuda.synchronize()
