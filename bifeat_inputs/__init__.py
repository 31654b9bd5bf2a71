"""Seeded synthetic inputs for the BiFeat feature-loading path.

This package produces *data only*: node-feature tables, graphs, sampled
minibatch blocks.  It holds none of the method's arithmetic (no quantizer, no
decoder, no aggregation) and is the one module that both the CPU oracle's
tests and the HIP path's tests/bench may import.

Everything is a pure function of (seed, coordinates), so any row of a table
that is far too large to materialise (hundreds of GB) can be produced anywhere,
bit-identically, on the host (numpy, here) and on the device
(``bifeat_inputs.device``, a small HIP generator with the same recipe).
"""
from .features import (column_params, feature_rows, feature_chunk, mix64,
                       stream_key, FeatureSpec)
from .graphs import UniformGraph, PowerLawGraph, sample_blocks, draw_seeds, Block, full_csr
from .workloads import WORKLOADS, Workload, make_graph, launch_set, two_round_set, BATCHES_PER_STEP

__all__ = [
    "column_params", "feature_rows", "feature_chunk", "mix64", "stream_key",
    "FeatureSpec", "UniformGraph", "PowerLawGraph", "sample_blocks",
    "draw_seeds", "Block", "full_csr", "WORKLOADS", "Workload", "make_graph", "launch_set", "two_round_set",
    "BATCHES_PER_STEP",
]
