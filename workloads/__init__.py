"""Seeded synthetic decode workloads (inputs only).

This package builds the tensors that both the CPU oracle and the HIP library
consume: queries, bf16 KV caches, sequence lengths, block tables and seeds.
It holds none of the method's arithmetic (no scores, no selection, no
sampling, no softmax); it only draws random numbers, rounds them to bf16 once
and lays them out.
"""
from .bf16 import f32_to_bf16_bits, bf16_bits_to_f32
from .configs import (
    Workload,
    make_workload,
    config1,
    config2,
    config3,
    config4,
    config5,
    small_gqa,
    to_paged,
    chunk_queries,
)

__all__ = [
    "f32_to_bf16_bits",
    "bf16_bits_to_f32",
    "Workload",
    "make_workload",
    "config1",
    "config2",
    "config3",
    "config4",
    "config5",
    "small_gqa",
    "to_paged",
    "chunk_queries",
]
