"""Seeded synthetic workloads (model shapes, random weights, prompts).

This package only draws random numbers and describes shapes.  It holds none of the
decoder / self-speculative-decoding arithmetic, so that both the CPU oracle and the
HIP library can be fed bit-identical inputs without sharing any method code.
"""
from .models import (WORKLOADS, ModelShape, Workload, make_weights, make_prompt,
                     weight_tensor_names, reduced_depth)

__all__ = ["WORKLOADS", "ModelShape", "Workload", "make_weights", "make_prompt",
           "weight_tensor_names", "reduced_depth"]
