"""Seeded synthetic inputs for the five Dolphin hot-path workloads.

This package holds input generators only: pseudo-random streams, the logits ->
probability preparation that a neural front-end would do, symbol tables of the
user functions, and upstream gradients.  It contains none of the arithmetic of
the Distribution operators or provenances; both the CPU oracle's tests and the
HIP library's tests/bench import it so that they see byte-identical inputs.
"""
from .gen import (  # noqa: F401
    splitmix64, uniform01, normal, softmax_rows, beta22, hashed_table,
    keep_mask, sum_table, grid_edges, grid_reach_triples, Workload,
    config1, config2, config3, config4, config5, make_config, CONFIG_NAMES,
    random_digraph, join_triples, closure_workload, product_stage_tables, product_workload, hwf_symbol_tables, hwf_workload, HWF_OPS,
)
