"""ctypes binding over the C ABI declared in include/ss.h.

Argument marshalling only: every step of the path (compression, convolution, epilogue) runs in
the HIP library.  PyTorch provides device memory and the stream.  There is no fallback: if the
library has not been built, importing fails with an instruction to build it.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

import torch

_HERE = Path(__file__).resolve().parent
LIB_PATH = _HERE / "libss.so"

SS_OK = 0
SS_ERR_INVALID_ARG, SS_ERR_BAD_MASK, SS_ERR_UNSUPPORTED, SS_ERR_WORKSPACE, SS_ERR_HIP = -1, -2, -3, -4, -5
SS_F16, SS_BF16, SS_I8, SS_F8 = 0, 1, 2, 3
SS_K_CRS, SS_K_RSC = 0, 1
SS_ACT_NONE, SS_ACT_RELU, SS_ACT_GELU = 0, 1, 2

EXPORTS = ["ss_status_string", "ss_packed_bytes", "ss_dense_bytes", "ss_mask_compress", "ss_mask_decompress",
           "ss_dense_pack", "ss_conv2d_workspace_bytes", "ss_conv2d_fwd", "ss_conv2d_dense_fwd",
           "ss_conv2d_res_fwd", "ss_conv2d_dense_res_fwd", "ss_mask_update_compress", "ss_maxpool2d", "ss_dwconv2d_fwd",
           "ss_conv2d_q8_fwd", "ss_conv2d_q8_dense_fwd", "ss_conv2d_pw_fused_fwd", "ss_conv2d_pw_fused_dense_fwd",
           "ss_weights_check", "ss_conv2d_fwd_static_ws", "ss_conv2d_pw_fused_query"]
DEBUG_EXPORTS = ["ss_debug_force_tile", "ss_debug_limit_blocks", "ss_debug_force_split", "ss_debug_issue_peak", "ss_debug_lds_bandwidth"]          # include/ss_debug.h: test hooks


class ss_weight_desc(ctypes.Structure):
    _fields_ = [("cout", ctypes.c_int32), ("cin", ctypes.c_int32), ("kh", ctypes.c_int32), ("kw", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("korder", ctypes.c_int32)]


class SSError(RuntimeError):
    def __init__(self, status: int, what: str, detail=None):
        self.status = status
        self.detail = detail
        super().__init__(f"{what}: {status_string(status)}" + (f" {detail}" if detail is not None else ""))


def _load() -> ctypes.CDLL:
    if not LIB_PATH.exists():
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
            "or python paper_2411_00288_amd/build.py). There is no CPU fallback.")
    lib = ctypes.CDLL(str(LIB_PATH))
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    dp = ctypes.POINTER(ss_weight_desc)
    lib.ss_status_string.restype = ctypes.c_char_p
    lib.ss_status_string.argtypes = [ctypes.c_int]
    lib.ss_packed_bytes.argtypes = [dp, ctypes.POINTER(sz)]
    lib.ss_dense_bytes.argtypes = [dp, ctypes.POINTER(sz)]
    lib.ss_mask_compress.argtypes = [dp, vp, vp, vp, ctypes.POINTER(i32), vp]
    lib.ss_mask_update_compress.argtypes = [dp, vp, vp, vp, vp, ctypes.POINTER(i32), vp]
    lib.ss_maxpool2d.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, i32, vp, vp]
    lib.ss_dwconv2d_fwd.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, i32, i32, i32, i32, i32, vp, vp]
    lib.ss_mask_decompress.argtypes = [dp, vp, vp, vp]
    lib.ss_dense_pack.argtypes = [dp, vp, vp, vp, vp]
    lib.ss_conv2d_workspace_bytes.argtypes = [dp, i32, i32, i32, i32, i32, i32, i32, ctypes.POINTER(sz)]
    conv_args = [dp, vp, i32, i32, i32, vp, vp, i32, i32, i32, i32, i32, vp, vp, sz, vp]
    lib.ss_conv2d_fwd.argtypes = conv_args
    lib.ss_conv2d_dense_fwd.argtypes = conv_args
    res_args = conv_args[:7] + [vp] + conv_args[7:]          # residual after bias
    lib.ss_conv2d_res_fwd.argtypes = res_args
    lib.ss_conv2d_dense_res_fwd.argtypes = res_args
    q8_args = [dp, vp, i32, i32, i32, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, sz, vp]
    lib.ss_conv2d_q8_fwd.argtypes = q8_args
    lib.ss_conv2d_q8_dense_fwd.argtypes = q8_args
    fused_args = [dp, vp, i32, i32, i32, vp, vp, i32, i32, i32, i32, i32, dp, vp, vp, vp, i32, vp, vp]
    lib.ss_conv2d_pw_fused_fwd.argtypes = fused_args
    lib.ss_conv2d_pw_fused_dense_fwd.argtypes = fused_args
    lib.ss_weights_check.argtypes = [dp, vp, i32, vp]
    lib.ss_conv2d_pw_fused_query.argtypes = [dp, i32, i32, i32, i32, dp, i32, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.ss_conv2d_fwd_static_ws.argtypes = conv_args[:13] + [vp]            # no workspace pair
    lib.ss_debug_force_tile.argtypes = [i32]
    lib.ss_debug_limit_blocks.argtypes = [i32]
    lib.ss_debug_force_split.argtypes = [i32]
    lib.ss_debug_issue_peak.argtypes = [i32, i32, vp, sz, ctypes.POINTER(ctypes.c_float), vp]
    lib.ss_debug_lds_bandwidth.argtypes = [i32, i32, i32, vp, sz, ctypes.POINTER(ctypes.c_float), vp]
    for name in EXPORTS[1:] + DEBUG_EXPORTS:
        getattr(lib, name).restype = ctypes.c_int
    return lib


_lib = _load()


def status_string(status: int) -> str:
    return _lib.ss_status_string(int(status)).decode()


def make_desc(cout, cin, kh, kw, dtype=SS_F16, korder=SS_K_CRS) -> ss_weight_desc:
    return ss_weight_desc(int(cout), int(cin), int(kh), int(kw), int(dtype), int(korder))


def _stream_ptr(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dev_ptr(t, name, dtypes=None, allow_none=False):
    if t is None:
        if allow_none:
            return None
        raise SSError(SS_ERR_INVALID_ARG, f"{name} is None")
    if not t.is_cuda:
        raise SSError(SS_ERR_INVALID_ARG, f"{name} must live in device memory")
    if not t.is_contiguous():
        raise SSError(SS_ERR_INVALID_ARG, f"{name} must be contiguous")
    if dtypes is not None and t.dtype not in dtypes:
        raise SSError(SS_ERR_INVALID_ARG, f"{name} has dtype {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


_T16 = (torch.float16, torch.bfloat16, torch.int16, torch.uint16)
_T8 = (torch.int8, torch.uint8, torch.float8_e4m3fn)


def _wtypes(desc):
    """Tensor dtypes accepted for weights of a descriptor."""
    return _T8 if desc.dtype in (SS_I8, SS_F8) else _T16


def torch_dtype(dtype: int):
    return {SS_F16: torch.float16, SS_BF16: torch.bfloat16, SS_I8: torch.int8, SS_F8: torch.uint8}[dtype]


def ss_packed_bytes(desc: ss_weight_desc) -> int:
    out = ctypes.c_size_t(0)
    st = _lib.ss_packed_bytes(ctypes.byref(desc), ctypes.byref(out))
    if st != SS_OK:
        raise SSError(st, "ss_packed_bytes")
    return int(out.value)


def ss_dense_bytes(desc: ss_weight_desc) -> int:
    out = ctypes.c_size_t(0)
    st = _lib.ss_dense_bytes(ctypes.byref(desc), ctypes.byref(out))
    if st != SS_OK:
        raise SSError(st, "ss_dense_bytes")
    return int(out.value)


def ss_mask_compress(desc: ss_weight_desc, W: torch.Tensor, M: torch.Tensor, packed: torch.Tensor | None = None,
                     stream=None) -> torch.Tensor:
    """W [cout, K] 16-bit, M [cout, K] uint8 (device) -> packed uint8 buffer (device)."""
    K = desc.cin * desc.kh * desc.kw
    if W is not None and W.numel() != desc.cout * K or M is not None and M.numel() != desc.cout * K:
        raise SSError(SS_ERR_INVALID_ARG, "ss_mask_compress: W/M size does not match the descriptor")
    if packed is None:
        packed = torch.empty(ss_packed_bytes(desc), dtype=torch.uint8, device=W.device)
    elif packed.numel() * packed.element_size() < ss_packed_bytes(desc):
        raise SSError(SS_ERR_INVALID_ARG, "ss_mask_compress: packed buffer too small")
    bad = (ctypes.c_int32 * 2)(-1, -1)
    st = _lib.ss_mask_compress(ctypes.byref(desc), _dev_ptr(W, "W", _wtypes(desc)), _dev_ptr(M, "M", (torch.uint8, torch.bool)),
                               _dev_ptr(packed, "packed"), bad, _stream_ptr(stream))
    if st != SS_OK:
        raise SSError(st, "ss_mask_compress", detail=(bad[0], bad[1]) if st == SS_ERR_BAD_MASK else None)
    return packed


def ss_mask_update_compress(desc: ss_weight_desc, W: torch.Tensor, U: torch.Tensor, M: torch.Tensor,
                            packed: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """W <- round16(W + U) in place, and packed <- compress(W, M): re-packing after a weight update."""
    K = desc.cin * desc.kh * desc.kw
    if W is None or U is None or M is None or W.numel() != desc.cout * K or U.numel() != desc.cout * K or \
            M.numel() != desc.cout * K or U.dtype != W.dtype:
        raise SSError(SS_ERR_INVALID_ARG, "ss_mask_update_compress: W/U/M do not match the descriptor")
    if packed is None:
        packed = torch.empty(ss_packed_bytes(desc), dtype=torch.uint8, device=W.device)
    elif packed.numel() * packed.element_size() < ss_packed_bytes(desc):
        raise SSError(SS_ERR_INVALID_ARG, "ss_mask_update_compress: packed buffer too small")
    bad = (ctypes.c_int32 * 2)(-1, -1)
    st = _lib.ss_mask_update_compress(ctypes.byref(desc), _dev_ptr(W, "W", _T16), _dev_ptr(U, "U", _T16),
                                      _dev_ptr(M, "M", (torch.uint8, torch.bool)), _dev_ptr(packed, "packed"), bad,
                                      _stream_ptr(stream))
    if st != SS_OK:
        raise SSError(st, "ss_mask_update_compress", detail=(bad[0], bad[1]) if st == SS_ERR_BAD_MASK else None)
    return packed


def ss_mask_decompress(desc: ss_weight_desc, packed: torch.Tensor, out: torch.Tensor | None = None,
                       stream=None) -> torch.Tensor:
    K = desc.cin * desc.kh * desc.kw
    if out is None:
        out = torch.empty((desc.cout, K), dtype=torch_dtype(desc.dtype), device=packed.device)
    st = _lib.ss_mask_decompress(ctypes.byref(desc), _dev_ptr(packed, "packed"), _dev_ptr(out, "out", _wtypes(desc)),
                                 _stream_ptr(stream))
    if st != SS_OK:
        raise SSError(st, "ss_mask_decompress")
    return out


def ss_dense_pack(desc: ss_weight_desc, W: torch.Tensor, M: torch.Tensor | None, dense: torch.Tensor | None = None,
                  stream=None) -> torch.Tensor:
    K = desc.cin * desc.kh * desc.kw
    if W.numel() != desc.cout * K or (M is not None and M.numel() != desc.cout * K):
        raise SSError(SS_ERR_INVALID_ARG, "ss_dense_pack: W/M size does not match the descriptor")
    if dense is None:
        dense = torch.empty(ss_dense_bytes(desc), dtype=torch.uint8, device=W.device)
    elif dense.numel() * dense.element_size() < ss_dense_bytes(desc):
        raise SSError(SS_ERR_INVALID_ARG, "ss_dense_pack: dense buffer too small")
    st = _lib.ss_dense_pack(ctypes.byref(desc), _dev_ptr(W, "W", _wtypes(desc)),
                            _dev_ptr(M, "M", (torch.uint8, torch.bool), allow_none=True),
                            _dev_ptr(dense, "dense"), _stream_ptr(stream))
    if st != SS_OK:
        raise SSError(st, "ss_dense_pack")
    return dense


def ss_weights_check(desc: ss_weight_desc, weights: torch.Tensor, sparse: bool = True, stream=None) -> None:
    """Raises unless `weights` was written for `desc` by the matching packing call (and, for the sparse form, with a
    valid mask).  One stream synchronisation; call once per buffer at set-up."""
    need = ss_packed_bytes(desc) if sparse else ss_dense_bytes(desc)
    if weights is None or weights.numel() * weights.element_size() < need:
        raise SSError(SS_ERR_INVALID_ARG, "ss_weights_check: buffer smaller than the descriptor's size query")
    st = _lib.ss_weights_check(ctypes.byref(desc), _dev_ptr(weights, "weights"), 1 if sparse else 0, _stream_ptr(stream))
    if st != SS_OK:
        raise SSError(st, "ss_weights_check")


def ss_debug_force_tile(tile_id: int) -> None:
    """Test hook (include/ss_debug.h): force the convolution kernels' tile variant; negative = library's choice."""
    _lib.ss_debug_force_tile(int(tile_id))


def ss_debug_limit_blocks(n: int) -> None:
    """Test hook (include/ss_debug.h): cap the workgroups of the resident-grid kernels; 0 = no cap."""
    _lib.ss_debug_limit_blocks(int(n))


def ss_debug_force_split(n: int) -> None:
    """Test hook (include/ss_debug.h): force the number of workgroups per output tile; 0 = the library decides."""
    _lib.ss_debug_force_split(int(n))


def ss_debug_issue_peak(dtype: int = SS_F16, sparse: bool = True, stream=None) -> float:
    """Calibration probe (include/ss_debug.h): register-only issue rate of the matrix instruction, dense-equivalent
    TFLOP/s."""
    scratch = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    out = ctypes.c_float(0.0)
    st = _lib.ss_debug_issue_peak(int(dtype), 1 if sparse else 0, _dev_ptr(scratch, "scratch"), scratch.numel(),
                                  ctypes.byref(out), _stream_ptr(stream))
    if st != SS_OK:
        raise SSError(st, "ss_debug_issue_peak")
    return float(out.value)


def ss_debug_lds_bandwidth(write: int, waves_per_simd: int, row_bytes: int = 592, stream=None) -> float:
    """Calibration probe (include/ss_debug.h): LDS bandwidth of one compute unit, GB/s."""
    scratch = torch.empty(2 << 20, dtype=torch.uint8, device="cuda")
    out = ctypes.c_float(0.0)
    st = _lib.ss_debug_lds_bandwidth(int(write), int(waves_per_simd), int(row_bytes), _dev_ptr(scratch, "scratch"),
                                     scratch.numel(), ctypes.byref(out), _stream_ptr(stream))
    if st != SS_OK:
        raise SSError(st, "ss_debug_lds_bandwidth")
    return float(out.value)


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def _check_operands(what, desc, wbuf, bias, sparse):
    """Sizes the asynchronous calls rely on and cannot check themselves: a short buffer would be read past its end."""
    need = ss_packed_bytes(desc) if sparse else ss_dense_bytes(desc)
    if _nbytes(wbuf) < need:
        raise SSError(SS_ERR_INVALID_ARG, f"{what}: weight buffer holds {_nbytes(wbuf)} bytes, the descriptor needs {need}")
    if bias is not None and bias.numel() < desc.cout:
        raise SSError(SS_ERR_INVALID_ARG, f"{what}: bias holds {bias.numel()} values, cout is {desc.cout}")


def ss_conv2d_workspace_bytes(desc, N, H, W, stride=(1, 1), pad=(0, 0)) -> int:
    out = ctypes.c_size_t(0)
    st = _lib.ss_conv2d_workspace_bytes(ctypes.byref(desc), N, H, W, stride[0], stride[1], pad[0], pad[1],
                                        ctypes.byref(out))
    if st != SS_OK:
        raise SSError(st, "ss_conv2d_workspace_bytes")
    return int(out.value)


def out_shape(desc, N, H, W, stride=(1, 1), pad=(0, 0)):
    if stride[0] <= 0 or stride[1] <= 0 or pad[0] < 0 or pad[1] < 0:
        raise SSError(SS_ERR_INVALID_ARG, "stride must be positive and pad non-negative")
    Ho = (H + 2 * pad[0] - desc.kh) // stride[0] + 1
    Wo = (W + 2 * pad[1] - desc.kw) // stride[1] + 1
    return (N, Ho, Wo, desc.cout)


def _conv_args(what, desc, x, wbuf, bias, stride, pad, act, y, workspace, stream, residual=None, with_res=False):
    if x is None or x.dim() != 4 or x.shape[3] != desc.cin:
        raise SSError(SS_ERR_INVALID_ARG, f"{what}: x must be NHWC with cin channels")
    N, H, W, _ = x.shape
    _check_operands(what, desc, wbuf, bias, "dense" not in what)
    shp = out_shape(desc, N, H, W, stride, pad)
    if shp[1] <= 0 or shp[2] <= 0:
        raise SSError(SS_ERR_INVALID_ARG, f"{what}: empty output")
    if y is None:
        y = torch.empty(shp, dtype=x.dtype, device=x.device)
    elif tuple(y.shape) != shp or y.dtype != x.dtype:
        raise SSError(SS_ERR_INVALID_ARG, f"{what}: y must be {shp} {x.dtype}")
    need = ss_conv2d_workspace_bytes(desc, N, H, W, stride, pad)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    if need > 0 and workspace is None:
        workspace = torch.zeros(need, dtype=torch.uint8, device=x.device)      # the ticket counters must start at zero
        ws_bytes = need
    if residual is not None and (tuple(residual.shape) != shp or residual.dtype != x.dtype or not residual.is_contiguous()):
        raise SSError(SS_ERR_INVALID_ARG, f"{what}: residual must be contiguous {shp} {x.dtype}")
    head = (ctypes.byref(desc), _dev_ptr(x, "x", (torch_dtype(desc.dtype),)), N, H, W, _dev_ptr(wbuf, "weights"),
            _dev_ptr(bias, "bias", (torch.float32,), allow_none=True))
    tail = (stride[0], stride[1], pad[0], pad[1], act,
            _dev_ptr(y, "y"), _dev_ptr(workspace, "workspace", allow_none=True), ws_bytes)
    args = head + ((_dev_ptr(residual, "residual", allow_none=True),) if with_res else ()) + tail
    return args, y, workspace


def _conv(fn, what, desc, x, wbuf, bias, stride, pad, act, y, workspace, stream, residual=None, with_res=False):
    args, y, _ws = _conv_args(what, desc, x, wbuf, bias, stride, pad, act, y, workspace, stream, residual, with_res)
    st = fn(*args, _stream_ptr(stream))
    if st != SS_OK:
        raise SSError(st, what)
    return y


def prepare_conv2d(desc, x, wbuf, bias=None, stride=(1, 1), pad=(0, 0), act=SS_ACT_NONE, y=None, workspace=None,
                   sparse=True, residual=None):
    """Marshal the arguments of ss_conv2d_fwd / ss_conv2d_dense_fwd (ss_conv2d_res_fwd / ss_conv2d_dense_res_fwd
    when a residual is given) once and return (launch, y):
    ``launch()`` enqueues the call on the current torch stream.  For launch-bound loops and graph
    capture, where per-call Python argument checking would dominate.  The tensors passed here
    must stay alive and in place for as long as ``launch`` is used."""
    with_res = residual is not None
    what = ("ss_conv2d_res_fwd" if sparse else "ss_conv2d_dense_res_fwd") if with_res else \
           ("ss_conv2d_fwd" if sparse else "ss_conv2d_dense_fwd")
    fn = getattr(_lib, what)
    args, y, ws = _conv_args(what, desc, x, wbuf, bias, stride, pad, act, y, workspace, None, residual, with_res)
    keep = (desc, x, wbuf, bias, y, ws, residual)

    def launch(_keep=keep):
        st = fn(*args, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        if st != SS_OK:
            raise SSError(st, what)
    return launch, y


def ss_conv2d_fwd(desc, x, packed, bias=None, stride=(1, 1), pad=(0, 0), act=SS_ACT_NONE, y=None, workspace=None,
                  stream=None) -> torch.Tensor:
    """2:4-sparse convolution: x NHWC [N,H,W,cin] -> y NHWC [N,Ho,Wo,cout] (same 16-bit dtype)."""
    return _conv(_lib.ss_conv2d_fwd, "ss_conv2d_fwd", desc, x, packed, bias, stride, pad, act, y, workspace, stream)


def ss_conv2d_fwd_static_ws(desc, x, packed, bias=None, stride=(1, 1), pad=(0, 0), act=SS_ACT_NONE, y=None,
                            stream=None) -> torch.Tensor:
    """ss_conv2d_fwd without a workspace argument: a split reduction's scratch is the library's own device array.
    `y` should be passed by callers that must not allocate (it is allocated here otherwise)."""
    what = "ss_conv2d_fwd_static_ws"
    if x is None or x.dim() != 4 or x.shape[3] != desc.cin:
        raise SSError(SS_ERR_INVALID_ARG, f"{what}: x must be NHWC with cin channels")
    N, H, W, _ = x.shape
    _check_operands(what, desc, packed, bias, True)
    shp = out_shape(desc, N, H, W, stride, pad)
    if shp[1] <= 0 or shp[2] <= 0:
        raise SSError(SS_ERR_INVALID_ARG, f"{what}: empty output")
    if y is None:
        y = torch.empty(shp, dtype=x.dtype, device=x.device)
    elif tuple(y.shape) != shp or y.dtype != x.dtype:
        raise SSError(SS_ERR_INVALID_ARG, f"{what}: y must be {shp} {x.dtype}")
    st = _lib.ss_conv2d_fwd_static_ws(ctypes.byref(desc), _dev_ptr(x, "x", (torch_dtype(desc.dtype),)), N, H, W,
                                      _dev_ptr(packed, "weights"), _dev_ptr(bias, "bias", (torch.float32,), allow_none=True),
                                      stride[0], stride[1], pad[0], pad[1], act, _dev_ptr(y, "y"), _stream_ptr(stream))
    if st != SS_OK:
        raise SSError(st, what)
    return y


def ss_conv2d_dense_fwd(desc, x, dense, bias=None, stride=(1, 1), pad=(0, 0), act=SS_ACT_NONE, y=None,
                        workspace=None, stream=None) -> torch.Tensor:
    """The dense-MFMA twin on the operand built by ss_dense_pack."""
    return _conv(_lib.ss_conv2d_dense_fwd, "ss_conv2d_dense_fwd", desc, x, dense, bias, stride, pad, act, y,
                 workspace, stream)


def ss_conv2d_res_fwd(desc, x, packed, bias=None, residual=None, stride=(1, 1), pad=(0, 0), act=SS_ACT_NONE, y=None,
                      workspace=None, stream=None) -> torch.Tensor:
    """2:4-sparse convolution closing a residual block: y = act(conv(x) + bias + residual), residual NHWC like y."""
    return _conv(_lib.ss_conv2d_res_fwd, "ss_conv2d_res_fwd", desc, x, packed, bias, stride, pad, act, y, workspace,
                 stream, residual, True)


def ss_conv2d_dense_res_fwd(desc, x, dense, bias=None, residual=None, stride=(1, 1), pad=(0, 0), act=SS_ACT_NONE,
                            y=None, workspace=None, stream=None) -> torch.Tensor:
    """The dense-MFMA twin of ss_conv2d_res_fwd."""
    return _conv(_lib.ss_conv2d_dense_res_fwd, "ss_conv2d_dense_res_fwd", desc, x, dense, bias, stride, pad, act, y,
                 workspace, stream, residual, True)


def _q8_args(what, desc, x, wbuf, scale, bias, stride, pad, act, y, workspace):
    if x is None or x.dim() != 4 or x.shape[3] != desc.cin:
        raise SSError(SS_ERR_INVALID_ARG, f"{what}: x must be NHWC with cin channels")
    N, H, W, _ = x.shape
    _check_operands(what, desc, wbuf, bias, "dense" not in what)
    if scale is not None and scale.numel() < desc.cout:
        raise SSError(SS_ERR_INVALID_ARG, f"{what}: scale holds {scale.numel()} values, cout is {desc.cout}")
    shp = out_shape(desc, N, H, W, stride, pad)
    if shp[1] <= 0 or shp[2] <= 0:
        raise SSError(SS_ERR_INVALID_ARG, f"{what}: empty output")
    if y is None:
        y = torch.empty(shp, dtype=torch.float16, device=x.device)
    elif tuple(y.shape) != shp or y.dtype != torch.float16:
        raise SSError(SS_ERR_INVALID_ARG, f"{what}: y must be {shp} float16")
    need = ss_conv2d_workspace_bytes(desc, N, H, W, stride, pad)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    if need > 0 and workspace is None:
        workspace = torch.zeros(need, dtype=torch.uint8, device=x.device)
        ws_bytes = need
    xtypes = (torch.int8,) if desc.dtype == SS_I8 else (torch.uint8, torch.float8_e4m3fn)
    args = (ctypes.byref(desc), _dev_ptr(x, "x", xtypes), N, H, W, _dev_ptr(wbuf, "weights"),
            _dev_ptr(scale, "scale", (torch.float32,), allow_none=True),
            _dev_ptr(bias, "bias", (torch.float32,), allow_none=True), stride[0], stride[1], pad[0], pad[1], act,
            SS_F16, _dev_ptr(y, "y"), _dev_ptr(workspace, "workspace", allow_none=True), ws_bytes)
    return args, y, workspace


def prepare_conv2d_q8(desc, x, wbuf, scale=None, bias=None, stride=(1, 1), pad=(0, 0), act=SS_ACT_NONE, y=None,
                      workspace=None, sparse=True):
    """prepare_conv2d for the 8-bit integer entry points: returns (launch, y)."""
    what = "ss_conv2d_q8_fwd" if sparse else "ss_conv2d_q8_dense_fwd"
    fn = getattr(_lib, what)
    args, y, ws = _q8_args(what, desc, x, wbuf, scale, bias, stride, pad, act, y, workspace)
    keep = (desc, x, wbuf, scale, bias, y, ws)

    def launch(_keep=keep):
        st = fn(*args, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        if st != SS_OK:
            raise SSError(st, what)
    return launch, y


def ss_conv2d_q8_fwd(desc, x, packed, scale=None, bias=None, stride=(1, 1), pad=(0, 0), act=SS_ACT_NONE, y=None,
                     workspace=None, stream=None) -> torch.Tensor:
    """2:4-sparse convolution on 8-bit operands (int8, or FP8 E4M3 bytes): x NHWC -> y NHWC float16 =
    act(scale * sum + bias)."""
    args, y, _ws = _q8_args("ss_conv2d_q8_fwd", desc, x, packed, scale, bias, stride, pad, act, y, workspace)
    st = _lib.ss_conv2d_q8_fwd(*args, _stream_ptr(stream))
    if st != SS_OK:
        raise SSError(st, "ss_conv2d_q8_fwd")
    return y


def ss_conv2d_q8_dense_fwd(desc, x, dense, scale=None, bias=None, stride=(1, 1), pad=(0, 0), act=SS_ACT_NONE, y=None,
                           workspace=None, stream=None) -> torch.Tensor:
    """The dense integer-MFMA twin of ss_conv2d_q8_fwd."""
    args, y, _ws = _q8_args("ss_conv2d_q8_dense_fwd", desc, x, dense, scale, bias, stride, pad, act, y, workspace)
    st = _lib.ss_conv2d_q8_dense_fwd(*args, _stream_ptr(stream))
    if st != SS_OK:
        raise SSError(st, "ss_conv2d_q8_dense_fwd")
    return y


def prepare_conv2d_pw_fused(desc1, x, w1, bias1, stride, pad, act1, desc2, w2, bias2=None, residual=None,
                            act2=SS_ACT_NONE, y=None, sparse=True):
    """Marshal the arguments of ss_conv2d_pw_fused_fwd / ss_conv2d_pw_fused_dense_fwd once; returns (launch, y)."""
    what = "ss_conv2d_pw_fused_fwd" if sparse else "ss_conv2d_pw_fused_dense_fwd"
    if x is None or x.dim() != 4 or x.shape[3] != desc1.cin:
        raise SSError(SS_ERR_INVALID_ARG, f"{what}: x must be NHWC with cin channels")
    N, H, W, _ = x.shape
    _check_operands(what, desc1, w1, bias1, sparse)
    _check_operands(what, desc2, w2, bias2, sparse)
    shp1 = out_shape(desc1, N, H, W, stride, pad)
    if shp1[1] <= 0 or shp1[2] <= 0:
        raise SSError(SS_ERR_INVALID_ARG, f"{what}: empty output")
    shp = (N, shp1[1], shp1[2], desc2.cout)
    if y is None:
        y = torch.empty(shp, dtype=x.dtype, device=x.device)
    elif tuple(y.shape) != shp or y.dtype != x.dtype:
        raise SSError(SS_ERR_INVALID_ARG, f"{what}: y must be {shp} {x.dtype}")
    if residual is not None and (tuple(residual.shape) != shp or residual.dtype != x.dtype or not residual.is_contiguous()):
        raise SSError(SS_ERR_INVALID_ARG, f"{what}: residual must be contiguous {shp} {x.dtype}")
    fn = getattr(_lib, what)
    args = (ctypes.byref(desc1), _dev_ptr(x, "x", (torch_dtype(desc1.dtype),)), N, H, W, _dev_ptr(w1, "weights 1"),
            _dev_ptr(bias1, "bias1", (torch.float32,), allow_none=True), stride[0], stride[1], pad[0], pad[1], act1,
            ctypes.byref(desc2), _dev_ptr(w2, "weights 2"), _dev_ptr(bias2, "bias2", (torch.float32,), allow_none=True),
            _dev_ptr(residual, "residual", allow_none=True), act2, _dev_ptr(y, "y"))
    keep = (desc1, desc2, x, w1, w2, bias1, bias2, residual, y)

    def launch(_keep=keep):
        st = fn(*args, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        if st != SS_OK:
            raise SSError(st, what)
    return launch, y


def ss_conv2d_pw_fused_query(desc1, stride, pad, desc2, sparse=True):
    """(supported, pays): would the fused entry point take this pair, and does the library expect it to beat two calls?"""
    sup, pays = ctypes.c_int32(0), ctypes.c_int32(0)
    st = _lib.ss_conv2d_pw_fused_query(ctypes.byref(desc1), stride[0], stride[1], pad[0], pad[1], ctypes.byref(desc2),
                                       1 if sparse else 0, ctypes.byref(sup), ctypes.byref(pays))
    if st != SS_OK:
        raise SSError(st, "ss_conv2d_pw_fused_query")
    return bool(sup.value), bool(pays.value)


def ss_conv2d_pw_fused_fwd(desc1, x, packed1, bias1, stride, pad, act1, desc2, packed2, bias2=None, residual=None,
                           act2=SS_ACT_NONE, y=None) -> torch.Tensor:
    """k x k masked convolution followed by a 1x1 masked convolution (+ residual), the intermediate kept on chip."""
    launch, y = prepare_conv2d_pw_fused(desc1, x, packed1, bias1, stride, pad, act1, desc2, packed2, bias2, residual,
                                        act2, y, sparse=True)
    launch()
    return y


def ss_conv2d_pw_fused_dense_fwd(desc1, x, dense1, bias1, stride, pad, act1, desc2, dense2, bias2=None, residual=None,
                                 act2=SS_ACT_NONE, y=None) -> torch.Tensor:
    """The dense twin of ss_conv2d_pw_fused_fwd."""
    launch, y = prepare_conv2d_pw_fused(desc1, x, dense1, bias1, stride, pad, act1, desc2, dense2, bias2, residual,
                                        act2, y, sparse=False)
    launch()
    return y


def ss_maxpool2d(x: torch.Tensor, k: int = 3, stride: int = 2, pad: int = 1, y: torch.Tensor | None = None,
                 stream=None) -> torch.Tensor:
    """NHWC max pooling of a 16-bit tensor (positions outside the image do not take part)."""
    if x is None or x.dim() != 4 or x.dtype not in _T16 or stride <= 0:
        raise SSError(SS_ERR_INVALID_ARG, "ss_maxpool2d: x must be a 16-bit NHWC tensor")
    N, H, W, C = x.shape
    shp = (N, (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1, C)
    if y is None:
        y = torch.empty(shp, dtype=x.dtype, device=x.device)
    elif tuple(y.shape) != shp or y.dtype != x.dtype:
        raise SSError(SS_ERR_INVALID_ARG, f"ss_maxpool2d: y must be {shp} {x.dtype}")
    st = _lib.ss_maxpool2d(_dev_ptr(x, "x"), N, H, W, C, SS_F16 if x.dtype == torch.float16 else SS_BF16, k, stride, pad,
                           _dev_ptr(y, "y"), _stream_ptr(stream))
    if st != SS_OK:
        raise SSError(st, "ss_maxpool2d")
    return y


def ss_dwconv2d_fwd(x: torch.Tensor, w: torch.Tensor, bias: torch.Tensor | None = None, pad=(0, 0), act=SS_ACT_NONE,
                    y: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """Depthwise convolution, stride 1: x NHWC 16-bit, w [kh, kw, C] of the same dtype -> y NHWC."""
    if x is None or w is None or x.dim() != 4 or w.dim() != 3 or w.shape[2] != x.shape[3] or w.dtype != x.dtype or \
            x.dtype not in (torch.float16, torch.bfloat16):
        raise SSError(SS_ERR_INVALID_ARG, "ss_dwconv2d_fwd: x must be NHWC 16-bit and w [kh, kw, C] of the same dtype")
    N, H, W, C = x.shape
    kh, kw = int(w.shape[0]), int(w.shape[1])
    shp = (N, H + 2 * pad[0] - kh + 1, W + 2 * pad[1] - kw + 1, C)
    if shp[1] <= 0 or shp[2] <= 0:
        raise SSError(SS_ERR_INVALID_ARG, "ss_dwconv2d_fwd: empty output")
    if y is None:
        y = torch.empty(shp, dtype=x.dtype, device=x.device)
    elif tuple(y.shape) != shp or y.dtype != x.dtype:
        raise SSError(SS_ERR_INVALID_ARG, f"ss_dwconv2d_fwd: y must be {shp} {x.dtype}")
    st = _lib.ss_dwconv2d_fwd(_dev_ptr(x, "x"), N, H, W, C, SS_F16 if x.dtype == torch.float16 else SS_BF16,
                              _dev_ptr(w, "w"), _dev_ptr(bias, "bias", (torch.float32,), allow_none=True), kh, kw,
                              pad[0], pad[1], act, _dev_ptr(y, "y"), _stream_ptr(stream))
    if st != SS_OK:
        raise SSError(st, "ss_dwconv2d_fwd")
    return y
