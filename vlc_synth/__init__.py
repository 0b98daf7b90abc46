"""Seeded synthetic inputs for the selective-recompute prefill path.

This module only *describes* workloads (shapes, segment layouts) and draws
random numbers.  It holds none of the method's arithmetic: no RoPE, no index
selection, no attention, no rounding to storage types.  Both the CPU oracle's
tests and the HIP path's tests/benchmark take their inputs from here, so the
two sides see identical data without sharing any computation.
"""
from .workloads import (Shape, Segment, Request, Workload, SHAPES, make_workload,
                        layer_weights, head_weights, grid_positions, embedding_rows, cached_kv,
                        sensitivity_table, normal_f32, WEIGHT_NAMES, profile_sample)

__all__ = ["Shape", "Segment", "Request", "Workload", "SHAPES", "make_workload",
           "layer_weights", "head_weights", "grid_positions", "embedding_rows", "cached_kv", "sensitivity_table",
           "normal_f32", "WEIGHT_NAMES", "profile_sample"]
