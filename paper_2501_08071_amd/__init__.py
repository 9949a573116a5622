"""Fused multi-head attention forward for MI355X (gfx950), behind a C-ABI library, and the two
memory-bound row kernels (softmax, rmsnorm) and the fused GEMM + LeakyReLU next to it.

`attn_fwd`, `attn_supported`, `attn_status_str` mirror the entry points of
``include/attn.h``, `softmax_rows_fwd`, `rmsnorm_fwd` those of ``include/rowops.h``,
`gemm_leakyrelu_fwd` that of ``include/gemm.h``, the `probe_*` measuring aids those of
``include/probe.h``; they are loaded
lazily so that the input generator can be imported on a machine without the HIP library.
"""
from . import inputs  # noqa: F401

__all__ = ["inputs", "attn_fwd", "attn_fwd_o16", "attn_supported", "attn_status_str", "softmax_rows_fwd", "rmsnorm_fwd", "gemm_leakyrelu_fwd", "lib"]


def __getattr__(name):
    if name in ("attn_fwd", "attn_fwd_raw", "attn_fwd_o16", "attn_fwd_o16_raw", "attn_supported", "attn_status_str", "attn_kernel_name",
                "attn_tile_rows", "attn_tile_keys", "attn_launch_rows", "probe_mfma", "probe_softmax_valu", "probe_l2_read", "probe_launch_floor_us", "probe_issue_share", "lib", "AttnError", "F16", "BF16",
                "softmax_rows_fwd", "softmax_rows_fwd_raw", "rmsnorm_fwd", "rmsnorm_fwd_raw", "rowops_path", "rowops_status_str",
                "RowopsError", "gemm_leakyrelu_fwd", "gemm_leakyrelu_fwd_raw", "gemm_path", "gemm_status_str", "GemmError"):
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
