"""Seeded synthetic workloads and accuracy metrics for the quantized-attention path.

This package holds no arithmetic of the attention method itself: it only draws
inputs and scores outputs, so both the CPU oracle's tests and the GPU path's
tests can share it without sharing any of the method.
"""
from .inputs import (CONFIGS, WorkloadSpec, spec_of, make_inputs, make_head, round_to_dtype,
                     to_torch, from_torch, flops, awkward_values)
from .metrics import cos_sim, rel_l1, rmse, max_abs_over_row_linf

__all__ = ["CONFIGS", "WorkloadSpec", "spec_of", "make_inputs", "make_head", "round_to_dtype",
           "to_torch", "from_torch", "flops", "awkward_values", "cos_sim", "rel_l1", "rmse",
           "max_abs_over_row_linf"]
