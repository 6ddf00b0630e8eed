"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

This package only *makes inputs* (item embeddings, the fixed-degree item graph,
MLP parameters, user vectors, entry points).  It contains none of the search or
scoring arithmetic: the oracle and the HIP library each implement that on their
own and never import one another.
"""
from .gen import (  # noqa: F401
    SEED_BASE,
    Config,
    PRESETS,
    layer_sizes,
    make_layers,
    make_workload,
    random_mlp,
    to_host,
    scaled,
)
from .locality import locality_rank  # noqa: F401
