"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This module only draws random numbers and lays out input arrays (event lists, edge
features, negative destinations, static embeddings, initial weights).  It contains none
of the model's arithmetic: no sampling, no time encoding, no GRU, no attention.
"""
from .graphs import (CONFIGS, ModelDims, dims_of, gen_graph, gen_negatives, gen_params, gen_static, gen_labels,
                     batches_of)
from .problems import make_problem, custom_problem, batch_np

__all__ = ["CONFIGS", "ModelDims", "dims_of", "gen_graph", "gen_negatives", "gen_params", "gen_labels",
           "gen_static", "batches_of", "make_problem", "custom_problem", "batch_np"]
