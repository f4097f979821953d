"""Seeded synthetic inputs for the decode hot path (KV caches, queries, append streams).

This package is the only code shared by the CPU oracle's tests and the HIP path's
tests/bench.  It draws random numbers and converts number formats; it contains none
of the method's arithmetic (no dot products, no softmax, no index construction).
Anything that needs scores (placing a threshold at an order statistic, planting keys
above a threshold) takes the scores as an argument from its caller.
"""
from .generators import (  # noqa: F401
    CONFIGS,
    KVCache,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    make_cache,
    make_local_cache,
    make_queries,
    make_append_stream,
    drift_queries,
    plant_rows,
    planted_positions,
    round_to_bf16,
    tau_for_count,
    tau_for_fraction,
)
