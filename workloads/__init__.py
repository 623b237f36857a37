"""Seeded synthetic inputs for the multi-LoRA batched linear layer.

This package only *draws inputs* (request batches, activations, backbone and
adapter weights) and converts between storage formats.  It contains none of
the layer's arithmetic, so the CPU oracle and the HIP path can both take their
inputs from it without sharing any code of the method itself.
"""
from .bits import bf16_bits_from_f32, f32_from_bf16_bits, to_f64
from .configs import (
    CONFIG_NAMES,
    Projection,
    Workload,
    make_workload,
    make_custom,
    same_adapter_decode,
)

__all__ = [
    "bf16_bits_from_f32",
    "f32_from_bf16_bits",
    "to_f64",
    "CONFIG_NAMES",
    "Projection",
    "Workload",
    "make_workload",
    "make_custom",
    "same_adapter_decode",
]
