"""MI355X (gfx950) library for batched autoregressive generation of a LLaMA-architecture decoder.

The product is the C-ABI shared library built from csrc/ (see include/rl_gen.h); this package is the
thin Python binding: argument marshalling only.  There is no CPU fallback: importing `binding`
without the built library raises.
"""
from .binding import (RlGenError, RlGenShape, Generator, lib, ops, param_count, kv_bytes, work_bytes,
                      validate_shape, precision_level, kv_block_scaled, KERNEL_CLASSES)

__all__ = ["RlGenError", "RlGenShape", "Generator", "lib", "ops", "param_count", "kv_bytes", "work_bytes",
           "validate_shape", "precision_level", "kv_block_scaled", "KERNEL_CLASSES"]
