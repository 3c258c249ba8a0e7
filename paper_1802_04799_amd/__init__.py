"""Python binding of libtvg: fused conv2d / depthwise conv2d for one MI355X (gfx950).

Argument marshalling only; every operator runs in the HIP kernels of
``libtvg.so`` (C ABI declared in ``include/tvg.h``).  PyTorch supplies device
memory and streams.  There is no CPU fallback: if the library is missing,
``load()`` raises.
"""
from .binding import (  # noqa: F401
    TVG_BF16, TVG_F32, TVG_RELU, TVG_STREAM_OUT, ConvDesc, TvgError, conv2d_fused, dwconv2d_fused, lib_path, load,
    maxpool2d_3x3s2, status_string, tvg_conv2d_fused, tvg_conv2d_workspace_size,
    tvg_dwconv2d_fused, tvg_dwconv2d_workspace_size, tvg_maxpool2d_3x3s2, tvg_version,
    KERNEL_NAMES, tvg_conv2d_get_plan, tvg_conv2d_set_tile, ConvKnobs, tvg_conv2d_set_knobs, tvg_conv2d_get_knobs,
    tvg_conv2d_fused_static, tvg_static_scratch_bytes, tvg_conv2d_prepack_size, tvg_conv2d_prepack,
    tvg_conv2d_fused_prepacked, tvg_probe_copy, tvg_probe_mfma,
    tvg_conv2d_fused_dual, TVG_CENTRE_TAP_ONLY,
    TensorLife, tvg_plan_arena, dwpw_fused, tvg_dwpw_fused, tvg_dwpw_one_kernel, tvg_dwpw_workspace_size,
)
