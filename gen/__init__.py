"""Seeded synthetic workloads for the mixed-bitwidth MoE layer.

Inputs only: shapes, seeds, random tensors and the per-expert bitwidth tables of the
five benchmark configurations. This module holds none of the method's arithmetic (no
quantization, no routing, no FFN), so that the CPU oracle and the GPU library can both
be fed from it without sharing any code of the method.

The paper's own workloads (Switch Transformers checkpoints on Xsum/SAMsum, Section 4.1,
Table "MoE models used in experiments") are not available; these tensors take the
models' shapes and stand in for them.
"""
from .synth import (MASTER_SEED, CONFIGS, Config, seed_for, normal, bitwidth_table,
                    expert_weights, router_weights, hidden, tiny_config)

__all__ = ["MASTER_SEED", "CONFIGS", "Config", "seed_for", "normal", "bitwidth_table",
           "expert_weights", "router_weights", "hidden", "tiny_config"]
