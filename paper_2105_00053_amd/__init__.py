"""Quire-exact posit matrix products, convolutions, conversions and SGD update on
MI355X (gfx950): Python binding of libpositnn_hip.so (see include/positnn.h)."""
from .binding import (  # noqa: F401
    F32, F64, P8, P16, P32, P8_1, P8_2, P10_1, P10_2, P12_1, P12_2, ConvDesc, PositError, conv_desc, conv_out_hw, load, posit_axpy, posit_conv2d_bwd_data,
    posit_conv2d_bwd_weight, posit_conv2d_fwd, posit_conv2d_workspace, posit_convert, posit_gemm, posit_gemm_static, posit_gemm_workspace,
    posit_round, posit_relu, posit_relu_bwd, posit_maxpool2d_fwd, posit_maxpool2d_bwd, posit_avgpool2d_fwd, posit_avgpool2d_bwd,
    posit_gemm_noquire, posit_conv2d_fwd_noquire, posit_conv2d_bwd_data_noquire, posit_conv2d_bwd_weight_noquire,
    posit_unary, posit_unary_bwd, posit_cross_entropy, posit_mse, posit_axpy_multi,
)
