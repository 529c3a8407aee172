"""CPU oracle (test infrastructure only; see ripple_oracle.py)."""
from .ripple_oracle import (GraphState, BatchRecord, aggregate, layer_forward, layer_rows, in_adjacency,
                            full_recompute, recompute_rows, affected_sets, max_rel_err)

__all__ = ["GraphState", "BatchRecord", "aggregate", "layer_forward", "layer_rows", "in_adjacency",
           "full_recompute", "recompute_rows", "affected_sets", "max_rel_err"]
