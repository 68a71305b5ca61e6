"""Seeded synthetic inputs for one ragged verification step.

This module only draws random numbers and lays them out; it holds none of the
verification arithmetic (no attention, no acceptance rule).  Both the CPU
oracle's tests and the HIP path's tests/bench take their inputs from here so
that the two sides see byte-identical tensors.

All arrays are host numpy arrays.  16-bit brain floats have no numpy dtype and
are carried as ``uint16`` bit patterns (``dtype == "bf16"``).
"""
from .verify_step import (  # noqa: F401
    CONFIGS,
    VerifyStep,
    make_verify_step,
    make_custom_step,
    policy_inputs,
    make_policy_step,
    attach_tree,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    to_f64,
    algorithmic_bytes,
    algorithmic_bytes_tree,
    tree_internal_nodes,
    tree_accept_bytes_walk_form,
    accept_bytes_skipping_form,
)
