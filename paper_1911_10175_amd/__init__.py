"""MI355X (gfx950) zero-skipping convolution passes for CNN training.

Thin ctypes binding over libst_conv.so (C ABI in include/st_conv.h).  Every step of the
computation runs in the library's HIP kernels; Python only marshals arguments.  PyTorch is
used by callers to own device memory and streams.
"""
from .binding import (ConvDesc, StConvError, ST_PASS_BWI, ST_PASS_BWI_AUTO, ST_PASS_BWW, ST_PASS_BWW_AUTO,
                      ST_PASS_BWW_DY, ST_PASS_FWD, ST_PASS_FWD_AUTO, lib_path, load_library, st_conv_bwi,
                      st_conv_bwi_auto, st_conv_bwi_dense, st_conv_bww, st_conv_bww_auto, st_conv_bww_dense,
                      st_conv_bww_dy, st_conv_fwd, st_conv_fwd_auto, st_conv_fwd_dense, st_conv_fwd_static, st_conv_kernel_name, st_probe_issue_rate, st_conv_version,
                      st_conv_sparse_threshold, st_conv_workspace_bytes, st_status_str)
from .layout import (pack_activations, pack_filters, unpack_activations, unpack_filters)

__all__ = [
    "ConvDesc", "StConvError", "ST_PASS_FWD", "ST_PASS_BWI", "ST_PASS_BWW", "ST_PASS_BWW_DY", "ST_PASS_BWW_AUTO",
    "ST_PASS_FWD_AUTO", "ST_PASS_BWI_AUTO", "lib_path", "load_library",
    "st_conv_fwd", "st_conv_fwd_dense", "st_conv_fwd_auto", "st_conv_fwd_static", "st_conv_bwi", "st_conv_bwi_dense", "st_conv_bwi_auto",
    "st_conv_bww", "st_conv_bww_dense", "st_conv_bww_dy", "st_conv_bww_auto", "st_conv_workspace_bytes",
    "st_conv_sparse_threshold", "st_status_str", "st_conv_version", "st_conv_kernel_name", "st_probe_issue_rate",
    "pack_activations", "unpack_activations", "pack_filters", "unpack_filters",
]
