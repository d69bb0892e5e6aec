"""Seeded synthetic workloads (inputs only).

This package produces the tensors that both the CPU oracle and the HIP library
consume: keys, values, queries, chunk boundary lists, budgets.  It contains no
abstract, score, selection or attention arithmetic.
"""
from .workloads import (  # noqa: F401
    BASE_SEED,
    CONFIGS,
    Case,
    make_case,
    make_boundaries,
    uniform_boundaries,
    pack_boundaries,
    make_desert_keys,
)
from .quant import quantize_store, tag_four_bit, make_quant_case, QuantCase  # noqa: F401
