"""CPU oracle for the HydraGNN hot path -- TEST INFRASTRUCTURE, not product code.

A plain, slow numpy implementation of what the GPU library computes: the brute-force radius graph,
the EGNN-style message-passing layer (forward and reverse mode), mean pooling and the per-source
energy / force heads of the two-level multi-task decoder (paper section "Two-level hierarchical MTL
architecture"; backbone named in section "Numerical Results"). Floating point is float64 except the
cutoff test of the neighbour list, which is evaluated in float32 with every operation rounded on its
own because the edge list must be reproducible bit for bit.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package. It shares
no code with the HIP path and never imports it.

Parity pins: every function here is pinned by tests/test_oracle_*.py against something other than
itself (a KD-tree from scipy, dense adjacency products, closed forms, symmetry invariants, central
finite differences). Nothing here can be pinned to values printed in the paper, because the paper
prints no intermediate value of this path: "parity unpinned" with respect to the paper's tables.
"""
from .neighbors import radius_graph, radius_graph_rows, image_range, transpose_plan  # noqa: F401
from .optim import adamw_step  # noqa: F401
from .model import (  # noqa: F401
    unpack_layer,
    unpack_heads,
    silu,
    dsilu,
    embed_fwd,
    embed_bwd,
    edge_rbf,
    edge_rbf_bwd,
    edge_geometry,
    edge_geometry_bwd,
    mp_layer_fwd,
    mp_layer_bwd,
    pool_fwd,
    pool_bwd,
    routing_plan,
    heads_fwd,
    heads_bwd,
    deep_head_shapes,
    unpack_deep_heads,
    heads_deep_fwd,
    heads_deep_bwd,
    step_fwd_bwd,
    conservative_forces,
)
