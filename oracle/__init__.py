"""CPU oracle for the Convolution op family and Softmax -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package; the product (paper_1801_08058_amd) never does.
"""
from .conv_oracle import (  # noqa: F401
    Attrs, build, out_shape, conv_fwd, conv_fwd_at, conv_bwd_data, conv_bwd_data_gather,
    conv_bwd_data_at, conv_bwd_filters, conv_bwd_filters_at, nchw_to_blocked16,
    blocked16_to_nchw, f32_to_bf16_bits_rne, bf16_bits_to_f64, max_normalised_error,
    relu_bwd_mask, bias_grad, conv_bwd_data_relu,
)
from .softmax_oracle import softmax, softmax_bwd  # noqa: F401
from .conv3d_oracle import (  # noqa: F401
    Attrs3, out_shape3, conv3d_fwd, conv3d_bwd_data, conv3d_bwd_filters, conv3d_fwd_at,
    conv3d_bwd_data_at, conv3d_bwd_filters_at,
)
