"""Seeded synthetic inputs for the HydraGNN hot path (structures, weights, upstream gradients).

This package draws random numbers and lays arrays out; it holds none of the model's arithmetic.
Both the CPU oracle's tests and the GPU tests / benchmark feed from it, so the two sides always see
the same bytes.
"""
from .structures import (  # noqa: F401
    Batch,
    make_molecule,
    make_crystal,
    make_cubic_bulk,
    concat_graphs,
)
from .configs import CONFIGS, make_config, small_mixed_batch  # noqa: F401
from .weights import (  # noqa: F401
    layer_weight_count,
    head_weight_count,
    LAYER_FIELDS,
    HEAD_FIELDS,
    layer_field_slices,
    head_field_slices,
    init_layer_weights,
    init_head_weights,
    deep_head_field_slices,
    deep_head_weight_count,
    init_deep_head_weights,
    init_embedding,
    upstream_grads,
    ZMAX,
)
from .problems import make_weights, problem_from_batch, problem_from_config, sub_batch, sub_problem  # noqa: F401
