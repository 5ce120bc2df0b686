"""Seeded synthetic gradient sets (shapes + value recipes) used by tests and the benchmark.

This package only draws random inputs.  It contains none of the method's
arithmetic (no selection, no error sums, no allocation): both the CPU oracle's
tests and the GPU library's tests feed on the arrays produced here.
"""
from .shapes import (mlp_shapes, resnet18_shapes, resnet50_shapes,
                     gpt2_small_shapes, llama_shapes, numel)
from .gen import (Workload, make_workload, ratio_grid, bandwidth_trace, sin2_bandwidth_trace,
                  budget_from_bandwidth, WORKLOADS)

__all__ = ["mlp_shapes", "resnet18_shapes", "resnet50_shapes", "gpt2_small_shapes",
           "llama_shapes", "numel", "Workload", "make_workload", "ratio_grid",
           "bandwidth_trace", "sin2_bandwidth_trace", "budget_from_bandwidth", "WORKLOADS"]
