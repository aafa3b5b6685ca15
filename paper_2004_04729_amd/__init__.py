"""MI355X-native dithered backprop (arXiv 2004.04729): NSD quantisation of the preactivation
gradient and the two sparse backward products, as hand-written gfx950 HIP kernels behind a C ABI.

The Python layer only marshals arguments; every step runs in the HIP library.  There is no CPU
fallback: importing :mod:`paper_2004_04729_amd.binding` fails loudly when the library is missing.
"""
from .binding import (  # noqa: F401
    DbpError, Stats, PATH_AUTO, PATH_MFMA, PATH_GATHER, PATH_TWO_PLANES, F32, I8,
    abi_version, status_string, format_layout, linear_workspace_bytes, conv2d_workspace_bytes,
    nsd_quantize, nsd_quantize_static, topk_workspace_bytes, topk_quantize, dithered_linear_backward, dithered_conv2d_backward,
    conv2d_grouped_workspace_bytes, dithered_conv2d_backward_grouped, conv2d_products_grouped,
    dense_linear_backward, dense_conv2d_backward, linear_products, conv2d_products,
    BIAS_PER_COLUMN, BIAS_PER_ROW_GROUP, step_size_workspace_bytes, step_size, nsd_quantize_ex,
    linear_layer_workspace_bytes, conv2d_layer_workspace_bytes,
    dithered_linear_layer_backward, dithered_conv2d_layer_backward,
    quantize_int8_workspace_bytes, quantize_int8, dithered_linear_backward_q8, dithered_conv2d_backward_q8,
    lib, lib_path,
)
