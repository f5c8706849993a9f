"""Seeded synthetic inputs for dynamic label propagation.

This package only *makes inputs* (graphs, seed sets, insertion batches).  It holds
none of the method's arithmetic: no label propagation, no frontier logic.  Both the
CPU oracle's tests and the GPU library's tests/benchmarks draw their inputs from
here, so that the two sides see bit-identical arrays.

The graphs stand in for the paper's similarity graphs (kNN graphs over embeddings,
"Experimental Setup / Datasets") and its Erdos-Renyi random graphs; the paper's
own datasets are not used anywhere.
"""
from .graphs import (  # noqa: F401
    BASE_SEED,
    Batch,
    Problem,
    edges_to_csr,
    knn_mixture,
    knn_mixture_batch,
    sbm,
    sbm_vertex_batch,
    sbm_edge_batch,
    chung_lu,
    chung_lu_vertex_batch,
    small_random,
    small_random_batch,
    clustered_batch,
    erdos_renyi_single_batch,
    CONFIGS,
    csr_with_batch,
    make_config,
)
