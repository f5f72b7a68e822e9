"""Seeded synthetic inputs and workload shapes.

This package holds no arithmetic of the contraction itself: it only draws
numbers and names shapes, so that both the CPU oracle's tests and the HIP
path's tests/bench can be fed identical bits.
"""
from .gen import (MASTER_SEED, uniform_f64, normal_f64, to_storage, widen,
                  tensor, int8_tensor, DTYPE_F32, DTYPE_BF16, DTYPE_F16, DTYPE_FP8_E4M3, DTYPE_FP8_E5M2)
from .configs import CONFIGS, EXTRA_CONFIGS, Workload, make_inputs
from .attention import (ATTENTION_CONFIGS, AttentionWorkload, make_attention_inputs,
                        INT8_CONFIGS, Int8Workload, make_int8_inputs)

__all__ = ["MASTER_SEED", "uniform_f64", "normal_f64", "to_storage", "widen",
           "tensor", "int8_tensor", "DTYPE_F32", "DTYPE_BF16", "DTYPE_F16", "DTYPE_FP8_E4M3", "DTYPE_FP8_E5M2", "CONFIGS", "EXTRA_CONFIGS",
           "Workload", "make_inputs", "ATTENTION_CONFIGS", "AttentionWorkload", "make_attention_inputs", "INT8_CONFIGS", "Int8Workload", "make_int8_inputs"]
