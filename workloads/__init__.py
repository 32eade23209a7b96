"""Seeded synthetic MoE-layer workloads.

This package only draws random tensors and lays them out; it holds none of the
layer's arithmetic (no gating, no routing, no expert FFN).  Both the CPU oracle
tests and the GPU tests / bench take their inputs from here so that the two
sides see bit-identical values.
"""
from .moe_workloads import (  # noqa: F401
    MoEWorkload,
    WORKLOADS,
    get_workload,
    make_inputs,
    build_slot_pool,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    block_expert_map,
    relayout_maps,
    shared_slots_of,
)
