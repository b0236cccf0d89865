"""Seeded synthetic workload generators.

This package only produces input arrays (token strings in CSR form, arrival
ticks, scheduler parameters).  It contains none of the scheduling method's
arithmetic: no prefix matching, no selection, no tree.  Both the CPU oracle's
tests and the GPU path's tests/benchmarks draw their inputs from here so that
the two sides always see byte-identical inputs.
"""
from .generators import (  # noqa: F401
    Prompts,
    Workload,
    Stream,
    concat_prompts,
    take_prompts,
    config0,
    config1,
    config2,
    config2_deep,
    config3,
    config4_stream,
    refill_arrivals,
    shuffled_queue,
    toy_example,
    random_small,
    SEED_BASE,
    VOCAB,
    K_LPM_ENDPOINT,
)
