"""Seeded synthetic inputs for the RevFFN block (shapes of the Qwen1.5-MoE-A2.7B
decoder layer the paper fine-tunes, section 4.1 "Base Model").

This module holds NO arithmetic of the method: it only names workload shapes,
draws Gaussian tensors in a fixed order, and rounds them to the storage dtype.
Both the fp64 CPU oracle and the HIP library are fed from here, so that the two
see bit-identical inputs.

The paper's real workload (instruction data pushed through pre-trained weights)
is not available offline; weights ~ N(0, 0.02^2), activations and upstream
gradients ~ N(0, 1) stand in for it.
"""
from .workloads import (WORKLOADS, Workload, make_inputs, make_weights, round_bf16,
                        bf16_bits, bits_to_f64, WEIGHT_FIELDS, weight_shapes,
                        ZIPF_ALPHA, zipf_router_bias)

__all__ = ["WORKLOADS", "Workload", "make_inputs", "make_weights", "round_bf16",
           "bf16_bits", "bits_to_f64", "WEIGHT_FIELDS", "weight_shapes",
           "ZIPF_ALPHA", "zipf_router_bias"]
