"""Device tile layout of the packed operands, as pure index arithmetic -- TEST INFRASTRUCTURE ONLY.

The GPU library stores the structured representation (Fig. 1 of the paper: kept values + 2-bit
indices) permuted into the register layout of gfx950's 32x32x32 sparse MFMA instruction.  That
permutation is a fixed bijection of the canonical form produced by ``oracle.compress``; this
module writes it out independently of the HIP sources so that ``packed_gpu`` can be compared
byte for byte with ``tile(canonical)``, and ``untile(packed_gpu)`` recovers the canonical arrays.

Layout (Mt = ceil(cout/32) row tiles, Ks = ceil(K/32) reduction steps, Kp = ceil(Ks/2)):
  header   64 x uint32 (256 bytes)
  values   [Mt][Ks][64 lanes][8 slots] uint16
           lane l, slot s  <->  row 32*mt + l%32,
                                block g = 8*ks + 4*(s//4) + 2*(l//32) + (s//2)%2,
                                element s%2 of the block's two kept values
  metadata [Mt][Kp][64 lanes] uint32; 16-bit half ks%2 of lane l holds nibble j = s//2
           (bits 4j..4j+3) = i0 | i1<<2 of the block in slots 2j, 2j+1
  padding rows / blocks: values 0, nibble 0x4
"""
from __future__ import annotations

import numpy as np

HEADER_BYTES = 256
MAGIC_SPARSE = 0x34325353
MAGIC_DENSE = 0x44325353
NO_BAD_BLOCK = 0xFFFFFFFF


def _dims(cout: int, K: int):
    Mt = -(-cout // 32)
    Ks = -(-K // 32)
    Kp = -(-Ks // 2)
    return Mt, Ks, Kp


def packed_bytes(cout: int, K: int) -> int:
    Mt, Ks, Kp = _dims(cout, K)
    return HEADER_BYTES + Mt * Ks * 1024 + Mt * Kp * 256


def dense_bytes(cout: int, K: int) -> int:
    Mt, Ks, _ = _dims(cout, K)
    return HEADER_BYTES + Mt * Ks * 2048


def header(magic, cout, cin, kh, kw, dtype, korder, first_bad=NO_BAD_BLOCK) -> np.ndarray:
    Mt, Ks, _ = _dims(cout, cin * kh * kw)
    h = np.zeros(64, dtype=np.uint32)
    h[:11] = [magic, 1, cout, cin, kh, kw, dtype, korder, Mt, Ks, first_bad]
    return h


def tile(vals: np.ndarray, meta: np.ndarray, *, cin, kh, kw, dtype, korder) -> np.ndarray:
    """Canonical (vals [cout,K/2] uint16, meta [cout,K/4] uint8) -> device bytes (uint8 array)."""
    cout, G = meta.shape
    K = 4 * G
    assert K == cin * kh * kw and vals.shape == (cout, 2 * G)
    Mt, Ks, Kp = _dims(cout, K)
    Gp = 8 * Ks
    # pad the canonical arrays to whole tiles
    vp = np.zeros((Mt * 32, Gp, 2), dtype=np.uint16)
    mp = np.full((Mt * 32, Gp), 0x4, dtype=np.uint32)
    vp[:cout, :G, :] = vals.reshape(cout, G, 2)
    mp[:cout, :G] = meta
    V = np.zeros((Mt, Ks, 64, 8), dtype=np.uint16)
    Md = np.zeros((Mt, Kp, 64), dtype=np.uint32)
    for l in range(64):
        rows = np.arange(Mt) * 32 + (l % 32)                       # [Mt]
        for s in range(8):
            g = 8 * np.arange(Ks) + 4 * (s // 4) + 2 * (l // 32) + (s // 2) % 2   # [Ks]
            V[:, :, l, s] = vp[rows[:, None], g[None, :], s % 2]
            if s % 2 == 0:
                j = s // 2
                nib = mp[rows[:, None], g[None, :]]                # [Mt, Ks]
                for ks in range(Ks):
                    Md[:, ks // 2, l] |= nib[:, ks] << np.uint32(4 * j + 16 * (ks % 2))
    if Ks % 2:   # the unused upper half of the last metadata tile is padding (nibble 0x4)
        Md[:, Kp - 1, :] |= np.uint32(0x44440000)
    out = np.concatenate([
        header(MAGIC_SPARSE, cout, cin, kh, kw, dtype, korder).view(np.uint8),
        V.reshape(-1).view(np.uint8),
        Md.reshape(-1).view(np.uint8),
    ])
    assert out.size == packed_bytes(cout, K)
    return out


def untile(packed: np.ndarray):
    """Device bytes -> (header uint32[64], vals [cout,K/2] uint16, meta [cout,K/4] uint8)."""
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    h = packed[:HEADER_BYTES].view(np.uint32).copy()
    cout, cin, kh, kw = (int(v) for v in h[2:6])
    K = cin * kh * kw
    G = K // 4
    Mt, Ks, Kp = _dims(cout, K)
    nv = Mt * Ks * 1024
    V = packed[HEADER_BYTES:HEADER_BYTES + nv].view(np.uint16).reshape(Mt, Ks, 64, 8)
    Md = packed[HEADER_BYTES + nv:HEADER_BYTES + nv + Mt * Kp * 256].view(np.uint32).reshape(Mt, Kp, 64)
    vals = np.zeros((cout, G, 2), dtype=np.uint16)
    meta = np.zeros((cout, G), dtype=np.uint8)
    for o in range(cout):
        mt, i = divmod(o, 32)
        for g in range(G):
            ks, gl = divmod(g, 8)
            s4, rem = divmod(gl, 4)        # s//4
            ga, pj = divmod(rem, 2)        # l//32, (s//2)%2
            l = 32 * ga + i
            s = 4 * s4 + 2 * pj
            vals[o, g, 0] = V[mt, ks, l, s]
            vals[o, g, 1] = V[mt, ks, l, s + 1]
            word = int(Md[mt, ks // 2, l]) >> (16 * (ks % 2))
            meta[o, g] = (word >> (4 * (s // 2))) & 0xF
    return h, vals.reshape(cout, 2 * G), meta


def tile_dense(Wm_bits: np.ndarray, *, cin, kh, kw, dtype, korder) -> np.ndarray:
    """Masked dense matrix M (.) W [cout, K] uint16 -> the dense twin's tiled operand bytes.

    Tile (mt, ks, h), lane l, slot s  <->  row 32*mt + l%32, k = 32*ks + 16*(l//32) + 8*h + s.
    """
    cout, K = Wm_bits.shape
    assert K == cin * kh * kw
    Mt, Ks, _ = _dims(cout, K)
    wp = np.zeros((Mt * 32, Ks * 32), dtype=np.uint16)
    wp[:cout, :K] = Wm_bits
    D = np.zeros((Mt, Ks, 2, 64, 8), dtype=np.uint16)
    for l in range(64):
        rows = np.arange(Mt) * 32 + (l % 32)
        for h in range(2):
            for s in range(8):
                k = 32 * np.arange(Ks) + 16 * (l // 32) + 8 * h + s
                D[:, :, h, l, s] = wp[rows[:, None], k[None, :]]
    out = np.concatenate([
        header(MAGIC_DENSE, cout, cin, kh, kw, dtype, korder).view(np.uint8),
        D.reshape(-1).view(np.uint8),
    ])
    assert out.size == dense_bytes(cout, K)
    return out


# ---------------------------------------------------------------------------------------------
# 8-bit integer operands (gfx950's 32x32x64 sparse and 32x32x32 dense integer MFMA)
#
# Mt = ceil(cout/32) row tiles, Ks = ceil(K/64) reduction steps of 64 indices (16 blocks):
#   values   [Mt][Ks][64 lanes][16 slots] bytes
#            lane l, slot s  <->  row 32*mt + l%32,
#                                 block g = 16*ks + 8*(s//8) + 4*(l//32) + (s%8)//2,
#                                 element s%2 of the block's two kept values
#   metadata [Mt][Ks][64 lanes] uint32: bits 4j..4j+3, j = s//2, = i0 | i1<<2 of the block in slots 2j, 2j+1
#   padding rows / blocks: values 0, nibble 0x4
# dense twin: tile (mt, ks, h), lane l, slot s (16 bytes)  <->  row 32*mt + l%32, k = 64*ks + 32*(l//32) + 16*h + s
# ---------------------------------------------------------------------------------------------
def _dims8(cout: int, K: int):
    return -(-cout // 32), -(-K // 64)


def packed_bytes8(cout: int, K: int) -> int:
    Mt, Ks = _dims8(cout, K)
    return HEADER_BYTES + Mt * Ks * 1024 + Mt * Ks * 256


def dense_bytes8(cout: int, K: int) -> int:
    Mt, Ks = _dims8(cout, K)
    return HEADER_BYTES + Mt * Ks * 2048


def header8(magic, cout, cin, kh, kw, korder, first_bad=NO_BAD_BLOCK) -> np.ndarray:
    Mt, Ks = _dims8(cout, cin * kh * kw)
    h = np.zeros(64, dtype=np.uint32)
    h[:11] = [magic, 1, cout, cin, kh, kw, 2, korder, Mt, Ks, first_bad]
    return h


def _block8(ks, l, s):
    return 16 * ks + 8 * (s // 8) + 4 * (l // 32) + (s % 8) // 2


def tile8(vals: np.ndarray, meta: np.ndarray, *, cin, kh, kw, korder) -> np.ndarray:
    """Canonical (vals [cout,K/2] int8, meta [cout,K/4] uint8) -> device bytes (uint8 array)."""
    cout, G = meta.shape
    K = 4 * G
    assert K == cin * kh * kw and vals.shape == (cout, 2 * G)
    Mt, Ks = _dims8(cout, K)
    Gp = 16 * Ks
    vp = np.zeros((Mt * 32, Gp, 2), dtype=np.uint8)
    mp = np.full((Mt * 32, Gp), 0x4, dtype=np.uint32)
    vp[:cout, :G, :] = vals.view(np.uint8).reshape(cout, G, 2)
    mp[:cout, :G] = meta
    V = np.zeros((Mt, Ks, 64, 16), dtype=np.uint8)
    Md = np.zeros((Mt, Ks, 64), dtype=np.uint32)
    ks = np.arange(Ks)
    for l in range(64):
        rows = np.arange(Mt) * 32 + (l % 32)
        for s in range(16):
            g = _block8(ks, l, s)
            V[:, :, l, s] = vp[rows[:, None], g[None, :], s % 2]
            if s % 2 == 0:
                Md[:, :, l] |= mp[rows[:, None], g[None, :]] << np.uint32(4 * (s // 2))
    out = np.concatenate([
        header8(MAGIC_SPARSE, cout, cin, kh, kw, korder).view(np.uint8),
        V.reshape(-1),
        Md.reshape(-1).view(np.uint8),
    ])
    assert out.size == packed_bytes8(cout, K)
    return out


def untile8(packed: np.ndarray):
    """Device bytes -> (header uint32[64], vals [cout,K/2] int8, meta [cout,K/4] uint8)."""
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    h = packed[:HEADER_BYTES].view(np.uint32).copy()
    cout, cin, kh, kw = (int(v) for v in h[2:6])
    K = cin * kh * kw
    G = K // 4
    Mt, Ks = _dims8(cout, K)
    nv = Mt * Ks * 1024
    V = packed[HEADER_BYTES:HEADER_BYTES + nv].reshape(Mt, Ks, 64, 16)
    Md = packed[HEADER_BYTES + nv:HEADER_BYTES + nv + Mt * Ks * 256].view(np.uint32).reshape(Mt, Ks, 64)
    vals = np.zeros((cout, G, 2), dtype=np.uint8)
    meta = np.zeros((cout, G), dtype=np.uint8)
    for o in range(cout):
        mt, i = divmod(o, 32)
        for g in range(G):
            ks, gl = divmod(g, 16)
            half, rem = divmod(gl, 8)      # s//8
            ga, pj = divmod(rem, 4)        # l//32, (s%8)//2
            l = 32 * ga + i
            s = 8 * half + 2 * pj
            vals[o, g, 0] = V[mt, ks, l, s]
            vals[o, g, 1] = V[mt, ks, l, s + 1]
            meta[o, g] = (int(Md[mt, ks, l]) >> (4 * (s // 2))) & 0xF
    return h, vals.reshape(cout, 2 * G).view(np.int8), meta


def tile_dense8(Wm: np.ndarray, *, cin, kh, kw, korder) -> np.ndarray:
    """Masked dense int8 matrix M (.) W [cout, K] -> the dense twin's tiled operand bytes."""
    cout, K = Wm.shape
    assert K == cin * kh * kw
    Mt, Ks = _dims8(cout, K)
    wp = np.zeros((Mt * 32, Ks * 64), dtype=np.uint8)
    wp[:cout, :K] = np.ascontiguousarray(Wm).view(np.uint8)
    D = np.zeros((Mt, Ks, 2, 64, 16), dtype=np.uint8)
    for l in range(64):
        rows = np.arange(Mt) * 32 + (l % 32)
        for h in range(2):
            for s in range(16):
                k = 64 * np.arange(Ks) + 32 * (l // 32) + 16 * h + s
                D[:, :, h, l, s] = wp[rows[:, None], k[None, :]]
    out = np.concatenate([header8(MAGIC_DENSE, cout, cin, kh, kw, korder).view(np.uint8), D.reshape(-1)])
    assert out.size == dense_bytes8(cout, K)
    return out
