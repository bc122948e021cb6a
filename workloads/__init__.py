"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path.

This package only *draws* inputs (graphs, feature stores, sampled mini-batches,
initial weights, labels) and converts storage formats.  It contains none of the
layer arithmetic: no projection, aggregation, fusion, sorting into CSR or
gradient code lives here.  Both `oracle/` and `paper_2408_08490_amd/` are free
to consume what it produces; it imports neither of them.
"""
from .synth import (  # noqa: F401
    Schema, HeteroGraph, Block, MiniBatch, LayerWeights,
    make_config, build_graph, sample_minibatch, init_weights,
    bf16_round, CONFIG_NAMES,
)
