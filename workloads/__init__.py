"""Seeded synthetic inputs and named workload presets.

This package is shared by the CPU oracle's tests and by the HIP path's
harness.  It holds no arithmetic of the method itself: it only draws
datasets, initial weights and hyper-parameter records.
"""
from .presets import PRESETS, preset, scaled_preset, param_count
from .methods import METHODS, method_preset
from .generate import make_inputs, make_split, to_bf16_bits, bf16_bits_to_f32

__all__ = ["METHODS", "method_preset", "PRESETS", "preset", "scaled_preset", "param_count",
           "make_inputs", "make_split", "to_bf16_bits", "bf16_bits_to_f32"]
