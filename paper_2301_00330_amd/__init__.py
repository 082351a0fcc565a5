"""Gradient-filtered convolution backward for AMD MI355X (gfx950).

``binding`` mirrors the C ABI of ``include/gf.h`` one to one; ``workloads`` holds
the layer tables and seeded synthetic inputs of the benchmark configurations.
All computation happens inside libgf.so (hand-written HIP kernels).
"""
from .binding import (ConvDesc, GfError, GF_BF16, GF_F32, GF_OK, GF_OP_BWD_EXACT,  # noqa: F401
                      GF_OP_BWD_FILTERED, gf_conv_bwd_filtered, GF_OP_BWD_CHAINED, gf_conv_bwd_chained, GF_OP_FILTER_SNR, gf_filter_grad_snr, gf_pool_activation_mask,
                      GF_OP_BWD_INPUT, GF_OP_BWD_WEIGHT, gf_conv_bwd_exact, gf_conv_bwd_input,
                      gf_conv_bwd_weight, gf_cost_model, gf_filter_grad, gf_out_shape,
                      gf_pool_activation, gf_version, gf_workspace_bytes, ptr,
                      GF_OP_BWD_WEIGHT_Q8, GF_OP_BWD_INPUT_Q8, gf_filter_grad_q8, gf_pool_activation_q8,
                      gf_kernel_sum_q8, gf_conv_bwd_weight_q8, gf_conv_bwd_input_q8)
