"""CPU oracle (test infrastructure only; see ripple_oracle.py)."""
from .ripple_oracle import (GraphState, BatchRecord, aggregate, layer_forward,
                            full_recompute, affected_sets, max_rel_err)

__all__ = ["GraphState", "BatchRecord", "aggregate", "layer_forward",
           "full_recompute", "affected_sets", "max_rel_err"]
