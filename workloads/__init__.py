"""Seeded synthetic inputs for batched hybrid KV-cache restoration.

This package only *draws* inputs (model shapes, random weights, token ids,
context lengths, page-pool churn scripts).  It holds none of the method's
arithmetic: no transformer math, no planner, no page allocator.  Both the CPU
oracle's tests and the HIP path's tests/bench take their inputs from here so
that the two sides see the same seeded data.
"""
from .shapes import ModelShape, SHAPES, shape_by_name
from .weights import WeightSource, bf16_round, bf16_bits, bits_to_f32
from .batches import (BatchSpec, make_batch, CONFIG_NAMES, churn_script,
                      hand_cost_model)

__all__ = [
    "ModelShape", "SHAPES", "shape_by_name", "WeightSource", "bf16_round",
    "bf16_bits", "bits_to_f32", "BatchSpec", "make_batch", "CONFIG_NAMES",
    "churn_script", "hand_cost_model",
]
