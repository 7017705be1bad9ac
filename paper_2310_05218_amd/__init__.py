"""Sliding Window Sum convolution and pooling for AMD Instinct MI355X (gfx950).

``binding`` wraps the C ABI of libswconv.so (``include/swconv.h``); ``inputs`` draws the seeded
synthetic workloads; ``build`` compiles the library with hipcc.  Importing the package loads
nothing: the library is opened on the first call.
"""
from .binding import (SW_POOL_AVG, SW_POOL_MAX, SwError, sw_conv1d, sw_conv2d, sw_conv2d_bias_relu,  # noqa: F401
                      sw_conv2d_depthwise, sw_conv2d_depthwise_bf16, sw_conv2d_depthwise_bias_relu, sw_conv2d_depthwise_dilated, sw_conv2d_depthwise_jit, sw_conv2d_depthwise_dilated_jit, sw_jit_prepare_depthwise_dilated, sw_jit_compile_check_dilated, sw_conv2d_dilated, sw_conv2d_s8, sw_conv2d_s8_nhwc, sw_conv2d_nhwc, sw_conv2d_bf16_nhwc, sw_conv2d_f16_nhwc, sw_dw_pw_block, sw_conv2d_s8_requant,
                      sw_jit_cached_kernels, sw_jit_compile_check, sw_jit_prepare_depthwise, sw_out_dim,
                      sw_pool1d, sw_pool2d, sw_version, sw_workspace_bytes, sw_out_dim_dilated, sw_last_kernel,
                      sw_s8_packed_filter_bytes, sw_s8_pack_filter, sw_conv2d_s8_packed, sw_probe,
                      SW_PROBE_MFMA_F32, SW_PROBE_MFMA_I8, SW_PROBE_FMA_F32, SW_PROBE_FMA_MFMA_F32, SW_PROBE_MFMA_F32_FED, SW_PROBE_MFMA_F32_FED2, SW_PROBE_MFMA_BF16)
