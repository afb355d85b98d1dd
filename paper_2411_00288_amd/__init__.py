"""2:4 semi-structured-sparse conv2d for AMD MI355X (gfx950).

``paper_2411_00288_amd.<name>`` for every entry point of include/ss.h (``ss_mask_compress``,
``ss_conv2d_fwd``, ``ss_conv2d_dense_fwd``, ...) resolves to the ctypes binding in ``binding.py``,
which is loaded on first use and raises if the HIP library has not been built: there is no
CPU fallback.  ``workloads`` (seeded synthetic inputs) is importable without the library.
"""
from __future__ import annotations

import importlib

_BINDING_NAMES = {
    "ss_status_string", "status_string", "ss_packed_bytes", "ss_dense_bytes", "ss_mask_compress", "ss_mask_update_compress", "ss_mask_decompress", "ss_maxpool2d", "ss_dwconv2d_fwd",
    "ss_dense_pack", "ss_conv2d_workspace_bytes", "ss_conv2d_fwd", "ss_conv2d_dense_fwd", "ss_conv2d_res_fwd",
    "ss_conv2d_dense_res_fwd", "make_desc", "out_shape", "prepare_conv2d",
    "ss_conv2d_q8_fwd", "ss_conv2d_q8_dense_fwd", "prepare_conv2d_q8", "SS_I8", "SS_F8", "ss_conv2d_pw_fused_fwd", "ss_conv2d_pw_fused_dense_fwd",
    "prepare_conv2d_pw_fused", "ss_weights_check", "ss_conv2d_pw_fused_query", "ss_conv2d_fwd_static_ws", "ss_debug_force_tile", "ss_debug_limit_blocks", "ss_debug_force_split", "ss_debug_issue_peak", "ss_debug_lds_bandwidth", "DEBUG_EXPORTS",
    "ss_weight_desc", "SSError", "torch_dtype", "EXPORTS", "LIB_PATH",
    "SS_OK", "SS_ERR_INVALID_ARG", "SS_ERR_BAD_MASK", "SS_ERR_UNSUPPORTED", "SS_ERR_WORKSPACE", "SS_ERR_HIP",
    "SS_F16", "SS_BF16", "SS_K_CRS", "SS_K_RSC", "SS_ACT_NONE", "SS_ACT_RELU", "SS_ACT_GELU",
}


def __getattr__(name):
    if name in _BINDING_NAMES or name == "binding":
        mod = importlib.import_module(".binding", __name__)
        if name == "binding":
            return mod
        if name == "ss_status_string":
            return mod.status_string
        return getattr(mod, name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")
