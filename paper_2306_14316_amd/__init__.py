"""MI355X (gfx950) im2win convolution: thin Python binding over libim2win.so.

The package only marshals arguments: every step of the path (the im2win
transform and the convolution over the im2win tensor) runs in the library's
HIP kernels.  PyTorch provides device memory and streams, nothing else.  There
is no CPU fallback: if the library is missing or no GPU is present, calls fail.
"""
from .binding import (  # noqa: F401
    Im2winError,
    conv2d_direct_fwd,
    conv2d_im2col_fwd,
    conv2d_im2win_fwd,
    conv2d_im2win_fwd_basic,
    conv2d_im2win_fwd_variant,
    conv2d_im2win_implicit_fwd,
    VARIANT_DEFAULT,
    VARIANT_NO_PIPELINE,
    VARIANT_NO_MFMA,
    VARIANT_NARROW_LOADS,
    VARIANT_SCALAR_LOADS,
    VARIANT_VALU_MICROKERNEL,
    PROBE_COPY,
    PROBE_NONTEMPORAL,
    PROBE_READ,
    PROBE_WRITE,
    conv2d_im2win_fwd_launch_info,
    im2win_probe_mfma_f32,
    im2win_probe_stream,
    im2win_transform_launch_info,
    im2col_footprint_bytes,
    im2col_transform,
    im2win_out_shape,
    im2win_transform,
    im2win_workspace_bytes,
    layer_sizes,
    lib_path,
    load_library,
    status_str,
)
