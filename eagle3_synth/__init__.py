"""Seeded synthetic inputs (weights, KV caches, features, trees, uniforms) and the
named workload shapes for the EAGLE-3 speculative step.

This package holds input synthesis only: a counter-based integer hash, table
look-ups and shape bookkeeping.  None of the method's arithmetic (norms, RoPE,
attention, GEMMs, top-k, acceptance) lives here, so both the CPU oracle's tests
and the GPU path's tests may draw the same bits from it.
"""
from .configs import Eagle3Shape, SHAPES, get_shape  # noqa: F401
from .inputs import (  # noqa: F401
    SEED, normal, uniform01, uniform_ints, make_d2t, TensorIds,
    layer_weights, target_globals, draft_weights, kv_layer, random_tree, reorder_tree, chain_tree, ragged_batch,
)
