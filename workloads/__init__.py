"""Seeded synthetic inputs for the CCE- loss (shapes, dtypes, id distributions).

This package holds input generation only: random hidden states, item tables,
target / negative ids, padding masks and their storage rounding.  It contains
none of the loss arithmetic, and it is the only code that both the fp64 CPU
oracle's tests and the HIP path's tests import.
"""
from .generators import (  # noqa: F401
    Workload,
    NEG_SHARED,
    NEG_PER_POSITION,
    NEG_FULL,
    BASE_SEED,
    CONFIG_NAMES,
    make_workload,
    config,
    bf16_bits_from_f32,
    f32_from_bf16_bits,
    zipf_ids,
    popularity_negatives,
    popularity_weights,
    alias_table,
)
