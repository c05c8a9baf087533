"""MI355X (gfx950) serving library for merged multi-task BERT models (arxiv 2107.05377, Section 3.3).

The compute path is the HIP shared library libmt_hip.so behind the C ABI declared in include/mt.h;
this package is its thin Python binding.  There is no CPU or PyTorch fallback.
"""
from .binding import (Model, MTError, make_config, pack_blob, lib, op_linear, op_linear_batched, op_attention, op_layernorm,
                      set_gemm_tile, mfma_peak, op_linear_sub, op_first_token_pool, op_linear_fp8, e4m3_quantize, KERNEL_CLASSES, EXPORTS, LIB_PATH,
                      MT_OK, MT_ERR_NULL, MT_ERR_CONFIG, MT_ERR_SHAPE, MT_ERR_STATE, MT_ERR_BLOB, MT_ERR_HIP,
                      MT_BF16, MT_FP32_CHECK, MT_FP8_FFN, MT_FP8_LAYER, MT_GELU_ERF, MT_GELU_TANH, MT_STATIC_SCRATCH_BYTES, mt_config, mt_task_desc)
from .synthetic import load_synthetic

__all__ = ["Model", "MTError", "make_config", "pack_blob", "lib", "op_linear", "op_linear_batched", "op_attention", "op_layernorm",
           "set_gemm_tile", "mfma_peak", "op_linear_sub", "op_first_token_pool", "load_synthetic", "KERNEL_CLASSES", "EXPORTS", "LIB_PATH"]
