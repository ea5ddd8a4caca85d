"""Seeded synthetic inputs and named workload presets.

This module is shared by the CPU oracle's tests, the GPU parity tests and the
benchmark.  It holds no part of the generation method's arithmetic: it only
names shapes and draws random weights / prompts from seeded generators.
"""
from .configs import ModelShape, Workload, PRESETS, LLAMA3_TABLE_SHAPES, preset
from .synth import make_weights, make_prompts, WEIGHT_ORDER, LAYER_TENSORS

__all__ = ["ModelShape", "Workload", "PRESETS", "LLAMA3_TABLE_SHAPES", "preset",
           "make_weights", "make_prompts", "WEIGHT_ORDER", "LAYER_TENSORS"]
