"""Seeded synthetic inputs for the minibatch feature gather.

This package only makes inputs: the power-law graph, the minibatch ID lists a
GraphSAGE-style sampler produces, the feature table and the hot-node list.  It
holds nothing of the gather itself (no dedup, no cache, no window, no
replacement policy), so both the HIP library's harness and the CPU oracle's
tests may draw their inputs from it.
"""
from .synth import (  # noqa: F401
    mix64, hash_chain, Graph, make_graph, hot_nodes, minibatch_seeds,
    sample_minibatch, layerwise_minibatch, normal_table, feature_rows, fill_store, TAGS, top_k_by_score,
)
from .configs import CONFIGS, Config, scaled  # noqa: F401
from . import native, synth  # noqa: F401,E402
