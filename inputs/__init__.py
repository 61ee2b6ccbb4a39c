"""Seeded synthetic workload generators shared by the CPU oracle's tests and the GPU path's tests."""
from .workloads import (CONFIGS, Inputs, Workload, as_float, bf16_bits_to_f32, config, custom,
                        f32_to_bf16_bits, generate, place_spans)

__all__ = ["CONFIGS", "Inputs", "Workload", "as_float", "bf16_bits_to_f32", "config", "custom",
           "f32_to_bf16_bits", "generate", "place_spans"]
