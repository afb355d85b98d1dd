"""CPU oracle for the 2:4 masked convolution -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``ss_oracle.c`` (plain C, fp64) plus the index-arithmetic description
of the device tile layout in ``device_layout.py``.  Only the tests, the smoke check and the
benchmark's CPU-baseline leg import this package; the GPU product path never does, and this
package imports nothing from the GPU package.

Paper passages followed: Sec. 3.1 Eq. (2) (mask validity), Fig. 1 (structured representation),
Sec. 3.3 Eq. (4) (direct convolution) and Eq. (6) (masked convolution).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "ss_oracle.c"
_LIB = _HERE / "libss_oracle.so"

F16, BF16, I8, F8 = 0, 1, 2, 3
K_CRS, K_RSC = 0, 1
ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2


def build(force: bool = False) -> Path:
    """Compile the C oracle with gcc (-O2, OpenMP).  Rebuilds when the source is newer."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", str(tmp), str(_SRC), "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_LIB))
        i64, p = ctypes.c_int64, ctypes.c_void_p
        lib.ss_oracle_bits_to_double.restype = ctypes.c_double
        lib.ss_oracle_bits_to_double.argtypes = [ctypes.c_uint16, ctypes.c_int]
        lib.ss_oracle_num_threads.restype = ctypes.c_int
        lib.ss_oracle_mask_check.restype = ctypes.c_int
        lib.ss_oracle_mask_check.argtypes = [p, i64, i64, p, p]
        lib.ss_oracle_compress.restype = ctypes.c_int
        lib.ss_oracle_compress.argtypes = [p, p, i64, i64, p, p]
        lib.ss_oracle_decompress.restype = None
        lib.ss_oracle_decompress.argtypes = [p, p, i64, i64, p]
        lib.ss_oracle_update.restype = None
        lib.ss_oracle_update.argtypes = [p, p, i64, ctypes.c_int]
        lib.ss_oracle_dwconv2d.restype = ctypes.c_int
        lib.ss_oracle_dwconv2d.argtypes = [p, i64, i64, i64, i64, ctypes.c_int, p, p, i64, i64, i64, i64, ctypes.c_int, p]
        lib.ss_oracle_maxpool2d.restype = ctypes.c_int
        lib.ss_oracle_maxpool2d.argtypes = [p, i64, i64, i64, i64, ctypes.c_int, i64, i64, i64, p]
        lib.ss_oracle_conv2d.restype = ctypes.c_int
        lib.ss_oracle_conv2d.argtypes = [p, i64, i64, i64, i64, p, p, i64, i64, i64,
                                         ctypes.c_int, ctypes.c_int, p, p, i64, i64, i64, i64,
                                         ctypes.c_int, p]
        lib.ss_oracle_conv2d_points.restype = ctypes.c_int
        lib.ss_oracle_conv2d_points.argtypes = [p, i64, i64, i64, i64, p, p, i64, i64, i64,
                                                ctypes.c_int, ctypes.c_int, p, p, i64, i64, i64, i64,
                                                ctypes.c_int, p, i64, p]
        lib.ss_oracle_compress8.restype = ctypes.c_int
        lib.ss_oracle_compress8.argtypes = [p, p, i64, i64, p, p]
        lib.ss_oracle_decompress8.restype = None
        lib.ss_oracle_decompress8.argtypes = [p, p, i64, i64, p]
        lib.ss_oracle_conv2d_q8.restype = ctypes.c_int
        lib.ss_oracle_conv2d_q8.argtypes = [p, i64, i64, i64, i64, p, p, i64, i64, i64, ctypes.c_int, p, p,
                                            i64, i64, i64, i64, ctypes.c_int, p]
        lib.ss_oracle_conv2d_q8_points.restype = ctypes.c_int
        lib.ss_oracle_conv2d_q8_points.argtypes = [p, i64, i64, i64, i64, p, p, i64, i64, i64, ctypes.c_int, p, p,
                                                   i64, i64, i64, i64, ctypes.c_int, p, i64, p]
        lib.ss_oracle_e4m3_to_double.restype = ctypes.c_double
        lib.ss_oracle_e4m3_to_double.argtypes = [ctypes.c_uint8]
        for fn in (lib.ss_oracle_conv2d_f8, lib.ss_oracle_conv2d_f8_points):
            fn.restype = ctypes.c_int
        lib.ss_oracle_conv2d_f8.argtypes = lib.ss_oracle_conv2d_q8.argtypes
        lib.ss_oracle_conv2d_f8_points.argtypes = lib.ss_oracle_conv2d_q8_points.argtypes
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def num_threads() -> int:
    return int(_load().ss_oracle_num_threads())


def bits_to_double(bits, dtype: int) -> np.ndarray:
    """Exact value of fp16 / bf16 bit patterns (uint16 array) as float64, via the C routine."""
    lib = _load()
    b = np.asarray(bits, dtype=np.uint16)
    out = np.empty(b.shape, dtype=np.float64)
    fb, fo = b.reshape(-1), out.reshape(-1)
    for i in range(fb.size):
        fo[i] = lib.ss_oracle_bits_to_double(int(fb[i]), dtype)
    return out


def mask_check(M) -> tuple[int, int, int]:
    """(status, row, group): status 0 = valid 2:4 mask, 1 = invalid block, 2 = K % 4 != 0."""
    M = _c(M, np.uint8)
    cout, K = M.shape
    r, g = ctypes.c_int64(-1), ctypes.c_int64(-1)
    st = _load().ss_oracle_mask_check(_ptr(M), cout, K, ctypes.byref(r), ctypes.byref(g))
    return int(st), int(r.value), int(g.value)


def compress(W_bits, M):
    """Canonical structured form: (vals uint16 [cout, K/2], meta uint8 [cout, K/4])."""
    W_bits, M = _c(W_bits, np.uint16), _c(M, np.uint8)
    cout, K = W_bits.shape
    assert M.shape == (cout, K)
    if K % 4:
        raise ValueError("K % 4 != 0")
    vals = np.zeros((cout, K // 2), dtype=np.uint16)
    meta = np.zeros((cout, K // 4), dtype=np.uint8)
    st = _load().ss_oracle_compress(_ptr(W_bits), _ptr(M), cout, K, _ptr(vals), _ptr(meta))
    if st:
        raise ValueError(f"invalid 2:4 mask (status {st})")
    return vals, meta


def decompress(vals, meta) -> np.ndarray:
    vals, meta = _c(vals, np.uint16), _c(meta, np.uint8)
    cout, G = meta.shape
    K = 4 * G
    out = np.empty((cout, K), dtype=np.uint16)
    _load().ss_oracle_decompress(_ptr(vals), _ptr(meta), cout, K, _ptr(out))
    return out


def update(W_bits, U_bits, dtype: int) -> np.ndarray:
    """V = round16(float(W) + float(U)) element-wise (binary32 sum, one rounding to the storage type)."""
    W_bits, U_bits = _c(W_bits, np.uint16).copy(), _c(U_bits, np.uint16)
    assert W_bits.shape == U_bits.shape
    _load().ss_oracle_update(_ptr(W_bits), _ptr(U_bits), W_bits.size, dtype)
    return W_bits


def _out_hw(H, Wd, kh, kw, stride, pad):
    return (H + 2 * pad[0] - kh) // stride[0] + 1, (Wd + 2 * pad[1] - kw) // stride[1] + 1


def conv2d(x_bits, W_bits, M, *, cin, kh, kw, korder=K_CRS, dtype=F16, bias=None,
           stride=(1, 1), pad=(0, 0), act=ACT_NONE, residual=None) -> np.ndarray:
    """Masked convolution, fp64, NHWC in / NHWC out, not rounded.  M=None: plain dense conv.
    residual: 16-bit patterns [N, Ho, Wo, cout] added before the activation."""
    x_bits, W_bits = _c(x_bits, np.uint16), _c(W_bits, np.uint16)
    N, H, Wd, c = x_bits.shape
    assert c == cin
    cout, K = W_bits.shape
    assert K == cin * kh * kw
    if M is not None:
        M = _c(M, np.uint8)
        assert M.shape == (cout, K)
    if bias is not None:
        bias = _c(bias, np.float32)
        assert bias.shape == (cout,)
    Ho, Wo = _out_hw(H, Wd, kh, kw, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise ValueError("empty output")
    if residual is not None:
        residual = _c(residual, np.uint16)
        assert residual.shape == (N, Ho, Wo, cout)
    y = np.empty((N, Ho, Wo, cout), dtype=np.float64)
    st = _load().ss_oracle_conv2d(_ptr(x_bits), N, H, Wd, cin, _ptr(W_bits), _ptr(M), cout, kh, kw,
                                  korder, dtype, _ptr(bias), _ptr(residual), stride[0], stride[1],
                                  pad[0], pad[1], act, _ptr(y))
    if st:
        raise ValueError(f"oracle conv2d failed (status {st})")
    return y


def conv2d_points(x_bits, W_bits, M, flat_idx, *, cin, kh, kw, korder=K_CRS, dtype=F16, bias=None,
                  stride=(1, 1), pad=(0, 0), act=ACT_NONE, residual=None) -> np.ndarray:
    """The same definition at sampled flat NHWC output indices only."""
    x_bits, W_bits = _c(x_bits, np.uint16), _c(W_bits, np.uint16)
    N, H, Wd, c = x_bits.shape
    assert c == cin
    cout, K = W_bits.shape
    if M is not None:
        M = _c(M, np.uint8)
    if bias is not None:
        bias = _c(bias, np.float32)
    flat_idx = _c(flat_idx, np.int64)
    Ho, Wo = _out_hw(H, Wd, kh, kw, stride, pad)
    assert flat_idx.min() >= 0 and flat_idx.max() < N * Ho * Wo * cout
    if residual is not None:
        residual = _c(residual, np.uint16)
        assert residual.shape == (N, Ho, Wo, cout)
    out = np.empty(flat_idx.shape, dtype=np.float64)
    st = _load().ss_oracle_conv2d_points(_ptr(x_bits), N, H, Wd, cin, _ptr(W_bits), _ptr(M), cout,
                                         kh, kw, korder, dtype, _ptr(bias), _ptr(residual), stride[0],
                                         stride[1], pad[0], pad[1], act, _ptr(flat_idx), flat_idx.size,
                                         _ptr(out))
    if st:
        raise ValueError(f"oracle conv2d_points failed (status {st})")
    return out


def maxpool2d(x_bits, *, dtype=F16, k=3, stride=2, pad=1) -> np.ndarray:
    """NHWC max pooling on 16-bit patterns; positions outside the image do not take part."""
    x_bits = _c(x_bits, np.uint16)
    N, H, Wd, C = x_bits.shape
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (Wd + 2 * pad - k) // stride + 1
    y = np.empty((N, Ho, Wo, C), dtype=np.uint16)
    st = _load().ss_oracle_maxpool2d(_ptr(x_bits), N, H, Wd, C, dtype, k, stride, pad, _ptr(y))
    if st:
        raise ValueError(f"oracle maxpool2d failed (status {st})")
    return y


def dwconv2d(x_bits, w_bits, *, dtype=F16, bias=None, pad=(0, 0), act=ACT_NONE) -> np.ndarray:
    """Depthwise convolution, stride 1: x NHWC, w [kh, kw, C] (16-bit patterns), fp64 result, not rounded."""
    x_bits, w_bits = _c(x_bits, np.uint16), _c(w_bits, np.uint16)
    N, H, Wd, C = x_bits.shape
    kh, kw, c2 = w_bits.shape
    assert c2 == C
    if bias is not None:
        bias = _c(bias, np.float32)
    Ho, Wo = H + 2 * pad[0] - kh + 1, Wd + 2 * pad[1] - kw + 1
    if Ho <= 0 or Wo <= 0:
        raise ValueError("empty output")
    y = np.empty((N, Ho, Wo, C), dtype=np.float64)
    st = _load().ss_oracle_dwconv2d(_ptr(x_bits), N, H, Wd, C, dtype, _ptr(w_bits), _ptr(bias), kh, kw, pad[0], pad[1],
                                    act, _ptr(y))
    if st:
        raise ValueError(f"oracle dwconv2d failed (status {st})")
    return y


# ---------------------------------------------------------------------------------------------
# 8-bit integer precision point
# ---------------------------------------------------------------------------------------------
def compress8(W_q, M):
    """Canonical structured form of an int8 matrix: (vals int8 [cout, K/2], meta uint8 [cout, K/4])."""
    W_q, M = _c(W_q, np.int8), _c(M, np.uint8)
    cout, K = W_q.shape
    assert M.shape == (cout, K)
    if K % 4:
        raise ValueError("K % 4 != 0")
    vals = np.zeros((cout, K // 2), dtype=np.int8)
    meta = np.zeros((cout, K // 4), dtype=np.uint8)
    st = _load().ss_oracle_compress8(_ptr(W_q), _ptr(M), cout, K, _ptr(vals), _ptr(meta))
    if st:
        raise ValueError(f"invalid 2:4 mask (status {st})")
    return vals, meta


def decompress8(vals, meta) -> np.ndarray:
    vals, meta = _c(vals, np.int8), _c(meta, np.uint8)
    cout, G = meta.shape
    out = np.empty((cout, 4 * G), dtype=np.int8)
    _load().ss_oracle_decompress8(_ptr(vals), _ptr(meta), cout, 4 * G, _ptr(out))
    return out


def _q8_args(x_q, W_q, M, scale, bias, cin, kh, kw):
    x_q, W_q = _c(x_q, np.int8), _c(W_q, np.int8)
    N, H, Wd, c = x_q.shape
    assert c == cin
    cout, K = W_q.shape
    assert K == cin * kh * kw
    if M is not None:
        M = _c(M, np.uint8)
        assert M.shape == (cout, K)
    if scale is not None:
        scale = _c(scale, np.float32)
        assert scale.shape == (cout,)
    if bias is not None:
        bias = _c(bias, np.float32)
        assert bias.shape == (cout,)
    return x_q, W_q, M, scale, bias, N, H, Wd, cout


def conv2d_q8(x_q, W_q, M, *, cin, kh, kw, korder=K_CRS, scale=None, bias=None, stride=(1, 1), pad=(0, 0),
              act=ACT_NONE) -> np.ndarray:
    """Integer masked convolution: exact int64 sums, then act(scale[o] * sum + bias[o]) in fp64, not rounded."""
    x_q, W_q, M, scale, bias, N, H, Wd, cout = _q8_args(x_q, W_q, M, scale, bias, cin, kh, kw)
    Ho, Wo = _out_hw(H, Wd, kh, kw, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise ValueError("empty output")
    y = np.empty((N, Ho, Wo, cout), dtype=np.float64)
    st = _load().ss_oracle_conv2d_q8(_ptr(x_q), N, H, Wd, cin, _ptr(W_q), _ptr(M), cout, kh, kw, korder, _ptr(scale),
                                     _ptr(bias), stride[0], stride[1], pad[0], pad[1], act, _ptr(y))
    if st:
        raise ValueError(f"oracle conv2d_q8 failed (status {st})")
    return y


def conv2d_q8_points(x_q, W_q, M, flat_idx, *, cin, kh, kw, korder=K_CRS, scale=None, bias=None, stride=(1, 1),
                     pad=(0, 0), act=ACT_NONE) -> np.ndarray:
    """The same definition at sampled flat NHWC output indices only."""
    x_q, W_q, M, scale, bias, N, H, Wd, cout = _q8_args(x_q, W_q, M, scale, bias, cin, kh, kw)
    flat_idx = _c(flat_idx, np.int64)
    Ho, Wo = _out_hw(H, Wd, kh, kw, stride, pad)
    assert flat_idx.min() >= 0 and flat_idx.max() < N * Ho * Wo * cout
    out = np.empty(flat_idx.shape, dtype=np.float64)
    st = _load().ss_oracle_conv2d_q8_points(_ptr(x_q), N, H, Wd, cin, _ptr(W_q), _ptr(M), cout, kh, kw, korder,
                                            _ptr(scale), _ptr(bias), stride[0], stride[1], pad[0], pad[1], act,
                                            _ptr(flat_idx), flat_idx.size, _ptr(out))
    if st:
        raise ValueError(f"oracle conv2d_q8_points failed (status {st})")
    return out


# ---------------------------------------------------------------------------------------------
# 8-bit float (OCP FP8 E4M3) precision point.  The structured representation of FP8 weights is the byte one above
# (compress8 / decompress8 on the bytes viewed as int8).
# ---------------------------------------------------------------------------------------------
def e4m3_to_double(b) -> np.ndarray:
    """Exact value of every E4M3 byte (NaN for 0x7F / 0xFF)."""
    b = np.ascontiguousarray(b, dtype=np.uint8)
    lib = _load()
    table = np.array([lib.ss_oracle_e4m3_to_double(i) for i in range(256)], dtype=np.float64)
    return table[b]


def _f8_args(x_b, W_b, M, scale, bias, cin, kh, kw):
    x_b, W_b = _c(x_b, np.uint8), _c(W_b, np.uint8)
    N, H, Wd, c = x_b.shape
    assert c == cin
    cout, K = W_b.shape
    assert K == cin * kh * kw
    if M is not None:
        M = _c(M, np.uint8)
        assert M.shape == (cout, K)
    if scale is not None:
        scale = _c(scale, np.float32)
        assert scale.shape == (cout,)
    if bias is not None:
        bias = _c(bias, np.float32)
        assert bias.shape == (cout,)
    return x_b, W_b, M, scale, bias, N, H, Wd, cout


def conv2d_f8(x_b, W_b, M, *, cin, kh, kw, korder=K_CRS, scale=None, bias=None, stride=(1, 1), pad=(0, 0),
              act=ACT_NONE) -> np.ndarray:
    """Masked convolution on E4M3 bytes: fp64 products and sums, then act(scale[o] * sum + bias[o]), not rounded."""
    x_b, W_b, M, scale, bias, N, H, Wd, cout = _f8_args(x_b, W_b, M, scale, bias, cin, kh, kw)
    Ho, Wo = _out_hw(H, Wd, kh, kw, stride, pad)
    if Ho <= 0 or Wo <= 0:
        raise ValueError("empty output")
    y = np.empty((N, Ho, Wo, cout), dtype=np.float64)
    st = _load().ss_oracle_conv2d_f8(_ptr(x_b), N, H, Wd, cin, _ptr(W_b), _ptr(M), cout, kh, kw, korder, _ptr(scale),
                                     _ptr(bias), stride[0], stride[1], pad[0], pad[1], act, _ptr(y))
    if st:
        raise ValueError(f"oracle conv2d_f8 failed (status {st})")
    return y


def conv2d_f8_points(x_b, W_b, M, flat_idx, *, cin, kh, kw, korder=K_CRS, scale=None, bias=None, stride=(1, 1),
                     pad=(0, 0), act=ACT_NONE) -> np.ndarray:
    x_b, W_b, M, scale, bias, N, H, Wd, cout = _f8_args(x_b, W_b, M, scale, bias, cin, kh, kw)
    flat_idx = _c(flat_idx, np.int64)
    Ho, Wo = _out_hw(H, Wd, kh, kw, stride, pad)
    assert flat_idx.min() >= 0 and flat_idx.max() < N * Ho * Wo * cout
    out = np.empty(flat_idx.shape, dtype=np.float64)
    st = _load().ss_oracle_conv2d_f8_points(_ptr(x_b), N, H, Wd, cin, _ptr(W_b), _ptr(M), cout, kh, kw, korder,
                                            _ptr(scale), _ptr(bias), stride[0], stride[1], pad[0], pad[1], act,
                                            _ptr(flat_idx), flat_idx.size, _ptr(out))
    if st:
        raise ValueError(f"oracle conv2d_f8_points failed (status {st})")
    return out
