"""Pins for the oracle's mask check / structured representation (Sec. 3.1 Eq. 2, Fig. 1).

None of these re-type the oracle's own code: they use closed forms (six patterns, their nibble
codes, byte counts), brute force over all patterns, inverse round trips and Lemma 3.3.
"""
import itertools

import numpy as np
import pytest

import oracle
from oracle import device_layout as dl
from paper_2411_00288_amd import workloads as wl

# closed form: the six 2-of-4 patterns and the nibble i0 | i1<<2 each must produce
PATTERN_NIBBLES = {(0, 1): 0x4, (0, 2): 0x8, (0, 3): 0xC, (1, 2): 0x9, (1, 3): 0xD, (2, 3): 0xE}


def test_exactly_six_patterns():
    # C(4,2) = 6 (the paper's printed formula (M-N)!/N! is garbled; the count of ways to pick
    # 2 of 4 without order is 6)
    pats = [p for p in itertools.product([0, 1], repeat=4) if sum(p) == 2]
    assert len(pats) == 6
    assert sorted(map(tuple, wl.PATTERNS.tolist())) == sorted(pats)
    # lexicographic order of kept positions
    kept = [tuple(np.flatnonzero(p)) for p in wl.PATTERNS]
    assert kept == sorted(kept) == list(PATTERN_NIBBLES)


def test_mask_check_accepts_all_patterns_rejects_everything_else():
    for bits in itertools.product([0, 1], repeat=4):
        st, r, g = oracle.mask_check(np.array([bits], dtype=np.uint8))
        assert (st == 0) == (sum(bits) == 2)
        if st:
            assert (st, r, g) == (1, 0, 0)
    # a 2 is not a bit
    assert oracle.mask_check(np.array([[2, 0, 0, 0]], dtype=np.uint8))[0] == 1
    # K not a multiple of 4
    assert oracle.mask_check(np.ones((1, 6), dtype=np.uint8))[0] == 2


def test_mask_check_reports_first_bad_block_row_major():
    M = np.tile(np.array([1, 1, 0, 0], dtype=np.uint8), (5, 6))
    M[3, 4 * 2 + 2] = 1      # row 3, group 2 -> three ones
    M[4, 0] = 0              # later row also bad
    assert oracle.mask_check(M) == (1, 3, 2)
    M[1, 4 * 5 + 0] = 0      # earlier row
    assert oracle.mask_check(M) == (1, 1, 5)


def test_groups_do_not_straddle_rows():
    # rows [1,1,1,0 | 0,0,0,1]... a mask valid only if blocks could straddle rows must be rejected
    M = np.array([[1, 1, 1, 0], [1, 0, 0, 0]], dtype=np.uint8)
    assert oracle.mask_check(M)[0] == 1


@pytest.mark.parametrize("kept,nibble", list(PATTERN_NIBBLES.items()))
def test_compress_single_block_brute_force(kept, nibble):
    W = np.array([[0x3C00, 0x4000, 0x4200, 0x4400]], dtype=np.uint16)   # 1, 2, 3, 4 in fp16
    M = np.zeros((1, 4), dtype=np.uint8)
    M[0, list(kept)] = 1
    vals, meta = oracle.compress(W, M)
    assert meta.tolist() == [[nibble]]
    assert vals.tolist() == [[W[0, kept[0]], W[0, kept[1]]]]
    back = oracle.decompress(vals, meta)
    assert back.tolist() == [(W[0] * M[0]).tolist()]


def test_compress_all_pattern_pairs_2x8():
    # brute force: every combination of patterns on a 2 x 8 matrix (6^4 = 1296 masks)
    W = (np.arange(16, dtype=np.uint16) + 0x3C01).reshape(2, 8)
    pats = list(PATTERN_NIBBLES)
    for combo in itertools.product(range(6), repeat=4):
        M = np.zeros((2, 8), dtype=np.uint8)
        for b, pid in enumerate(combo):
            r, g = divmod(b, 2)
            M[r, 4 * g + np.array(pats[pid])] = 1
        vals, meta = oracle.compress(W, M)
        exp_meta = np.array([PATTERN_NIBBLES[pats[p]] for p in combo], dtype=np.uint8).reshape(2, 2)
        assert np.array_equal(meta, exp_meta)
        assert np.array_equal(vals.reshape(-1), W[M == 1])          # row-major ascending positions
        assert np.array_equal(oracle.decompress(vals, meta), W * M)


def test_only_six_nibble_values_occur_and_round_trip_is_bit_exact():
    L = wl.Layer("t", N=1, H=4, W=4, cin=32, cout=24, kh=3, kw=3, pad=1, mask="logits", seed=5)
    d = wl.make_inputs(L)
    W = d["W"].copy()
    # plant special bit patterns among the weights: -0, NaN, inf, subnormal must survive bit for bit
    W[0, :8] = [0x8000, 0x7E01, 0x7C00, 0x0001, 0xFC00, 0x8001, 0x0000, 0xFFFF]
    vals, meta = oracle.compress(W, d["M"])
    assert set(np.unique(meta).tolist()) <= set(PATTERN_NIBBLES.values())
    back = oracle.decompress(vals, meta)
    expect = np.where(d["M"] == 1, W, 0).astype(np.uint16)
    assert np.array_equal(back, expect)
    # at most two non-zeros per block after decompression
    assert ((back.reshape(24, -1, 4) != 0).sum(-1) <= 2).all()
    # inputs untouched
    assert np.array_equal(W[1:], d["W"][1:])


def test_compress_rejects_invalid_mask():
    W = np.zeros((2, 8), dtype=np.uint16)
    M = np.tile(np.array([1, 1, 0, 0], dtype=np.uint8), (2, 2))
    M[1, 5] = 0
    with pytest.raises(ValueError):
        oracle.compress(W, M)


def test_storage_is_nine_sixteenths_of_dense():
    # Fig. 1: "roughly half the space": 16-bit values at half the count + one nibble per block
    cout, K = 64, 576
    vals_bytes = cout * (K // 2) * 2
    meta_bytes = cout * (K // 4) // 2          # 4 bits per block
    assert (vals_bytes + meta_bytes) * 16 == 9 * (cout * K * 2)
    # the device layout adds only the 256-byte header when cout % 32 == 0 and K % 64 == 0
    assert dl.packed_bytes(cout, K) == 256 + vals_bytes + meta_bytes
    assert dl.dense_bytes(cout, K) == 256 + cout * K * 2


def test_lemma_3_3_masking_as_additive_perturbation():
    # ||(M - 1) (.) W||_inf <= ||W||_inf (max absolute row sum), and M (.) W = W + dW exactly
    L = wl.Layer("t", N=1, H=2, W=2, cin=16, cout=8, kh=3, kw=3, pad=1, mask="top2", seed=2)
    d = wl.make_inputs(L)
    Wf = wl.from_bits(d["W"], L.dtype).astype(np.float64)
    vals, meta = oracle.compress(d["W"], d["M"])
    Wm = wl.from_bits(oracle.decompress(vals, meta), L.dtype).astype(np.float64)
    dW = Wm - Wf
    assert np.abs(dW).sum(1).max() <= np.abs(Wf).sum(1).max()
    assert np.array_equal(Wf + dW, Wm)
    # tight: the bound is attained when every kept entry is zero
    Wz = Wf.copy()
    Wz[d["M"] == 1] = 0
    assert np.abs((d["M"].astype(np.float64) - 1) * Wz).sum(1).max() == np.abs(Wz).sum(1).max()


@pytest.mark.parametrize("cout,cin,kh,kw", [(32, 16, 1, 1), (40, 8, 3, 3), (7, 4, 1, 1), (96, 24, 2, 2), (33, 96, 1, 1)])
def test_device_tiling_is_a_bijection_of_the_canonical_form(cout, cin, kh, kw):
    L = wl.Layer("t", N=1, H=4, W=4, cin=cin, cout=cout, kh=kh, kw=kw, mask="logits", seed=11)
    d = wl.make_inputs(L)
    vals, meta = oracle.compress(d["W"], d["M"])
    packed = dl.tile(vals, meta, cin=cin, kh=kh, kw=kw, dtype=L.dtype, korder=L.korder)
    assert packed.size == dl.packed_bytes(cout, L.K)
    h, v2, m2 = dl.untile(packed)
    assert h[0] == dl.MAGIC_SPARSE and h[2] == cout and h[10] == dl.NO_BAD_BLOCK
    assert np.array_equal(v2, vals) and np.array_equal(m2, meta)
    # every stored value appears exactly once: multiset of non-padding values is preserved
    Mt, Ks = -(-cout // 32), -(-L.K // 32)
    body = packed[256:256 + Mt * Ks * 1024].view(np.uint16)
    assert np.array_equal(np.sort(body[body != 0]), np.sort(vals[vals != 0].reshape(-1)))
    # metadata region holds only valid nibbles
    md = packed[256 + Mt * Ks * 1024:]
    nibs = np.concatenate([md & 0xF, md >> 4])
    assert set(np.unique(nibs).tolist()) <= set(PATTERN_NIBBLES.values())


def test_device_tiling_position_spot_checks():
    # hand-computed positions from the layout statement: row o, block g -> (tile, lane, slot)
    cout, cin = 64, 64           # K = 64, Ks = 2, Mt = 2
    vals = np.arange(cout * 32, dtype=np.uint16).reshape(cout, 32) + 1
    meta = np.full((cout, 16), 0x4, dtype=np.uint8)
    meta[37, 11] = 0xE
    packed = dl.tile(vals, meta, cin=cin, kh=1, kw=1, dtype=0, korder=0)
    V = packed[256:256 + 2 * 2 * 1024].view(np.uint16).reshape(2, 2, 64, 8)
    # row 37 -> mt 1, i 5.  block 11 -> ks 1, local block 3 = 4*0 + 2*1 + 1 -> lane 32+5, slots 2,3
    assert V[1, 1, 37, 2] == vals[37, 22] and V[1, 1, 37, 3] == vals[37, 23]
    # row 3, block 4 -> ks 0, local 4 = 4*1 + 0 + 0 -> lane 3, slots 4,5
    assert V[0, 0, 3, 4] == vals[3, 8] and V[0, 0, 3, 5] == vals[3, 9]
    Md = packed[256 + 4096:].view(np.uint32).reshape(2, 1, 64)
    # block 11 of row 37: ks=1 -> high half, nibble index 1 (slots 2,3) of lane 37
    assert (int(Md[1, 0, 37]) >> (16 + 4)) & 0xF == 0xE
    assert (int(Md[1, 0, 37]) & 0xFFFF) == 0x4444
