"""Seeded synthetic inputs for the Orthrus dual-view decode step.

This package only *produces data*: workload shapes, random tensors, page tables and
planted consensus cases.  It contains none of the method's arithmetic (no attention,
no softmax, no argmax, no accept rule), so that the CPU oracle and the HIP path can
both be fed from it without sharing any of the computation under test.
"""
from .configs import Workload, WORKLOADS, get_workload
from .generate import (
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    make_cache,
    make_block,
    make_consensus_case,
    make_sampling_case,
    make_step_inputs,
)

__all__ = [
    "Workload", "WORKLOADS", "get_workload", "f32_to_bf16_bits", "bf16_bits_to_f32",
    "make_cache", "make_block", "make_consensus_case", "make_sampling_case", "make_step_inputs",
]
