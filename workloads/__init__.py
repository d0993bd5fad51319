"""Seeded synthetic workloads shared by the CPU oracle, the tests and the benchmark.

This package holds workload descriptions (shapes, hyper-parameters) and seeded generators
for weights (a NumPy generator, and an integer hash that gives the same bits on the host and on the GPU), LoRA
factors, token ids, labels and sequence lengths.  It contains none of the method's
arithmetic: no forward pass, no noise transform, no estimator, no update.
"""
from .configs import Workload, WORKLOADS, get_workload, lora_layout, LoraTensor
from .generate import (make_frozen_weights, make_lora_masters, make_tokens, make_labels, make_lengths,
                       to_bf16_values)
from .hashed import make_frozen_weights_hashed, hashed_normal, hashed_levels

__all__ = ["Workload", "WORKLOADS", "get_workload", "lora_layout", "LoraTensor",
           "make_frozen_weights", "make_lora_masters", "make_tokens", "make_labels", "make_lengths",
           "to_bf16_values", "make_frozen_weights_hashed", "hashed_normal", "hashed_levels"]
