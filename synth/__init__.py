"""Seeded synthetic workloads (inputs only; none of the retrieval method's arithmetic lives here)."""
from .generator import (  # noqa: F401
    CONFIGS,
    Workload,
    GateWeights,
    make_centres,
    make_gate_weights,
    make_decomposed_gate_weights,
    item_chunk,
    make_items,
    make_queries,
    make_item_seeds,
    make_gen_mlp,
    ITEM_CHUNK,
)
