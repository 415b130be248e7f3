"""Seeded synthetic inputs (graphs, features, weights) shared by the tests, the
benchmark and the smoke check.

This package holds input generation only: it contains none of the CBM method's
arithmetic (no products, no compression, no normalisation) and imports neither
the CPU oracle nor the HIP library.
"""
from .graphs import (  # noqa: F401
    CONFIGS,
    BASE_SEED,
    Graph,
    make_graph,
    csr_from_edges,
    tiny_graph,
    citation_graph,
    collaboration_graph,
    protein_graph,
    rmat_graph,
)
from .features import (  # noqa: F401
    gaussian_features,
    integer_features,
    glorot_uniform,
)
