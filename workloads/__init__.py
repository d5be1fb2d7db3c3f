"""Seeded synthetic inputs shared by the tests, the oracle checks and the bench.

This package only *draws* tensors (random numbers, the planted low-rank
structure of K, dtype casts, the offline adapter fit).  It contains none of the
decode-step arithmetic: no projection of K or q, no scoring, no grouping, no
top-k, no attention.
"""
from .gen import (  # noqa: F401
    Config,
    PRESETS,
    LayerInputs,
    make_layer,
    make_problem_kv,
    make_q,
    fit_adapter,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    storage_to_f32,
    budget_to_groups,
)
