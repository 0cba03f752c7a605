"""Seeded synthetic decode-step batches (integers + bf16 bit patterns).

This package only *draws inputs*: sequence lengths, branch structure, block
tables and N(0,1) values rounded to bf16.  It contains none of the attention
arithmetic and no knowledge of how a KV page is laid out inside; both the CPU
oracle and the HIP library consume what it produces.
"""
from .generators import (  # noqa: F401
    AttnShape,
    Batch,
    BatchStructure,
    SegmentedStructure,
    reduce_structure,
    CONFIG_SEED_BASE,
    bf16_bits_from_f32,
    f32_from_bf16_bits,
    build_structure,
    compact_rows,
    fill_values_numpy,
    make_config,
    structure_config1,
    structure_config2,
    structure_config3,
    structure_config4,
    structure_config5,
    structure_wide,
    structure_custom,
    subset_rows,
)
