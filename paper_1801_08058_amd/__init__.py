"""MI355X (gfx950) Convolution op family behind a C ABI (include/ngconv.h).

The package holds the HIP sources (csrc/), their build script and a ctypes binding with
the same names as the C entry points.  Importing it requires the built library.
"""
from .binding import *  # noqa: F401,F403
from .binding import (  # noqa: F401
    ngc_conv_desc, make_desc, NgcError, LIB_PATH, EXPORTS,
    ngc_conv_out_shape, ngc_conv_workspace_bytes, ngc_conv_fwd, ngc_conv_bwd_data,
    ngc_conv_bwd_data_relu, ngc_conv_bwd_data_relu_db, ngc_bias_grad, ngc_softmax, ngc_softmax_bwd, ngc_softmax_variant,
    ngc_conv_bwd_filters, ngc_layout_convert, ngc_filter_convert, ngc_data_elems,
    ngc_filter_elems, ngc_conv_variant, ngc_status_string,
    ngc_conv3d_desc, make_desc3, ngc_conv3d_out_shape, ngc_conv3d_workspace_bytes, ngc_conv3d_fwd, ngc_conv3d_bwd_data,
    ngc_conv3d_bwd_filters, ngc_conv3d_filter_convert, ngc_conv3d_filter_elems, ngc_conv3d_data_elems, ngc_conv3d_variant,
    ngc_conv3d_bwd_data_relu, ngc_conv3d_bwd_data_relu_db, ngc_conv3d_bias_grad,
)
