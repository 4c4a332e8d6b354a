"""Seeded synthetic inputs for the PillarAttn hot path.

This package only draws random tensors and lays them out in a paged KV pool.
It holds none of the method's arithmetic (no attention, no softmax, no
selection): both the CPU oracle's tests and the HIP path's tests consume the
same arrays it returns.
"""
from .workloads import (CONFIGS, Workload, make_workload, make_custom,
                        bf16_bits_from_f32, f32_from_bf16_bits,
                        e4m3_bits_from_f32)

__all__ = ["CONFIGS", "Workload", "make_workload", "make_custom",
           "bf16_bits_from_f32", "f32_from_bf16_bits", "e4m3_bits_from_f32"]
