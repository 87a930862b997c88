"""MI355X-native hot path of adaptive-batch-size local gradient methods.

Thin ctypes binding over the C ABI in include/abs.h (libabs.so, built in-tree by
__graft_entry__.build()).  PyTorch is used only for device memory and the stream.
There is no CPU fallback: without the built library every call raises.
"""
from .binding import (Replicas, TestResult, average_bf16, average_bf16_static, copy_probe, layer_stats, load_library,
                      lr_linear_scaling, lr_schedule, next_batch_size, AbsError)

__all__ = ["Replicas", "TestResult", "average_bf16", "average_bf16_static", "copy_probe", "layer_stats", "load_library", "lr_linear_scaling",
           "lr_schedule",
           "next_batch_size", "AbsError"]
