"""Seeded synthetic LVLM-shaped inputs (Q, K, V, probe positions, tau).

This module only draws random tensors and rounds them to the storage dtype.
It holds none of the method's arithmetic and imports neither the CPU oracle
nor the HIP library; both are fed from here.
"""
from .generators import (CONFIGS, WorkloadSpec, Workload, make_workload,
                         make_custom, make_stack_layer_device, hybrid_probes, round_to_bf16, bf16_bits, base_seed)

__all__ = ["CONFIGS", "WorkloadSpec", "Workload", "make_workload",
           "make_custom", "make_stack_layer_device", "hybrid_probes", "round_to_bf16", "bf16_bits", "base_seed"]
