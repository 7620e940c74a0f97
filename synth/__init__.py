"""Seeded synthetic inputs shared by the oracle tests and the HIP path's tests/bench.

This package only *produces inputs* (tensor shape lists and seeded values).  It holds none of the
optimizer, packing or casting arithmetic of the method, and imports neither the oracle nor the
HIP binding.
"""
from .rng import normal_f32, normal_bf16, hash64_np  # noqa: F401
from .workloads import (  # noqa: F401
    TensorSpec, gpt_tensor_list, moe_tensor_list, moe_active_tensors, tensor_offsets, WORKLOADS,
)
