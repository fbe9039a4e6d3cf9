"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package only draws random numbers, rounds them to bf16 storage and lays out
index tables.  None of the restoration arithmetic (normalisation, projection,
rotary embedding, paging) lives here; the two implementations under test receive
the same buffers from these generators and share nothing else.
"""
from .bf16 import f32_to_bf16_bits, bf16_bits_to_f32, bf16_bits_to_f64
from .workloads import (
    Workload,
    WORKLOADS,
    BASE_SEED,
    layer_weights,
    layer_affine,
    layer_hidden,
    block_table,
    ragged_lengths,
    ragged_block_tables,
    dense_model_weights,
    batching_schedule,
)

__all__ = [
    "f32_to_bf16_bits",
    "bf16_bits_to_f32",
    "bf16_bits_to_f64",
    "Workload",
    "WORKLOADS",
    "BASE_SEED",
    "layer_weights",
    "layer_affine",
    "layer_hidden",
    "block_table",
    "ragged_lengths",
    "ragged_block_tables",
    "dense_model_weights",
    "batching_schedule",
]
