"""Seeded synthetic inputs (graphs, features, labels, weights) shared by every consumer.

This package only *draws data*.  It contains none of the method's arithmetic: no
normalisation, no aggregation, no partitioning.  Both the CPU oracle's tests and the
GPU path's tests/bench take their inputs from here so that they see identical bytes.
"""
from .graphs import rmat_graph, csr_from_edges, CONFIGS, make_config  # noqa: F401
from .tensors import attention_vectors, features, labels_and_mask, glorot_weights, to_bf16_grid  # noqa: F401
