"""Python access to the CPU oracle of the merged multi-task forward pass (test infrastructure only).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this package; the GPU
library never does.  The arithmetic lives in mt_oracle.c (C, float32 storage, float64 accumulation)
and, independently, in brute_tiny.py (scalar float64 loops for tiny shapes).
"""
from .binding import (Oracle, overhead, linear, layernorm, gelu, softmax_row, attention,
                      encoder_layer, layer_param_count, num_threads, set_num_threads)

__all__ = ["Oracle", "overhead", "linear", "layernorm", "gelu", "softmax_row", "attention",
           "encoder_layer", "layer_param_count", "num_threads", "set_num_threads"]
