"""MI355X-native Bolt hot path: FP16 MFMA GEMM / implicit-GEMM conv with fused epilogues,
persistent back-to-back fusion, channel padding and the light-weight tuner, behind libbolt.so.

The Python layer only marshals arguments; importing it fails if the HIP library is not built.
"""
from . import binding
from .binding import (ACT, LAYOUT_KN, LAYOUT_NK, OP_B2B_CONV, OP_B2B_CONV_RES, OP_B2B_GEMM, OP_B2B_GEMM_RES, OP_CONV2D, OP_CONV_CHAIN3, OP_GEMM, OP_GEMM_CHAIN3, BoltConfig, BoltError,
                      ConvDesc, GemmDesc, TENSOR_NCHW, TENSOR_NHWC, TuneResult, conv_desc, conv_out_hw, gemm_desc)

# the C ABI's entry points under their own names
bolt_gemm_epilogue = binding.gemm_epilogue
bolt_conv2d_fprop_nhwc = binding.conv2d_fprop_nhwc
bolt_gemm_epilogue_noalloc = binding.gemm_epilogue_noalloc
bolt_gemm_epilogue_residual = binding.gemm_epilogue_residual
bolt_conv2d_fprop_nhwc_residual = binding.conv2d_fprop_nhwc_residual
bolt_b2b_gemm = binding.b2b_gemm
bolt_b2b_conv = binding.b2b_conv
bolt_b2b_gemm_residual = binding.b2b_gemm_residual
bolt_b2b_conv_residual = binding.b2b_conv_residual
bolt_tune = binding.tune
bolt_b2b_gemm_chain = binding.b2b_gemm_chain
bolt_b2b_conv_chain = binding.b2b_conv_chain
bolt_b2b_gemm_chain_residual = binding.b2b_gemm_chain_residual
bolt_b2b_conv_chain_residual = binding.b2b_conv_chain_residual
bolt_tune_chain = binding.tune_chain
bolt_check_chain = binding.check_chain
bolt_chain_instance_supports = binding.chain_instance_supports
bolt_pad_channels_nhwc = binding.pad_channels_nhwc
bolt_nchw_to_nhwc = binding.nchw_to_nhwc
bolt_nhwc_to_nchw = binding.nhwc_to_nchw
bolt_bias_act = binding.bias_act
bolt_workspace_bytes = binding.workspace_bytes
bolt_check = binding.check
bolt_status_string = binding.status_string
bolt_num_instances = binding.num_instances
bolt_instance_config = binding.instance_config
bolt_instance_supports = binding.instance_supports
bolt_probe_mfma_peak = binding.probe_mfma_peak
bolt_probe_copy_bandwidth = binding.probe_copy_bandwidth
