"""Seeded synthetic inputs (graphs, features, labels, weights) shared by every consumer.

This package only *draws data*.  It contains none of the method's arithmetic: no
normalisation, no aggregation, no partitioning.  Both the CPU oracle's tests and the
GPU path's tests/bench take their inputs from here so that they see identical bytes.
"""
from .graphs import (rmat_graph, rmat_graph_counter, normal_counter, csr_from_edges, CONFIGS,  # noqa: F401
                     make_config)
from .tensors import attention_vectors, features, labels_and_mask, glorot_weights, to_bf16_grid  # noqa: F401
