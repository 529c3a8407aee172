"""Seeded synthetic inputs shared by the tests, the benchmark and both
implementations' callers.

This module only draws random numbers and keeps track of which edges and
vertices exist so that the update stream it emits is valid. It contains none
of the method's arithmetic (no aggregation, no layer math, no affected-set
logic) and imports neither the oracle nor the GPU package.

The graphs stand in for the paper's datasets (Table 2: Arxiv 169K/1.2M,
Products 2.5M/123.7M, Reddit 233K/114.6M) of which only the shapes are taken:
vertex and edge counts, feature width, class count. The update mix replaces the paper's
LinkBench-derived mix (Sec. 6.1.2), which is not available.
"""
from .graphs import (PowerLaw, degree_laws, chung_lu_graph, features, edge_weights, CONFIGS, get_config,
                     OP_EDGE_ADD, OP_EDGE_DEL, OP_VERTEX_ADD, OP_VERTEX_DEL,
                     OP_FEAT_UPDATE, OP_EDGE_REWEIGHT)
from .models import make_model, glorot
from .updates import UpdateStream
from .producer import BatchProducer

__all__ = ["PowerLaw", "degree_laws", "chung_lu_graph", "BatchProducer", "features", "edge_weights", "CONFIGS", "get_config",
           "make_model", "glorot", "UpdateStream",
           "OP_EDGE_ADD", "OP_EDGE_DEL", "OP_VERTEX_ADD", "OP_VERTEX_DEL",
           "OP_FEAT_UPDATE", "OP_EDGE_REWEIGHT"]
