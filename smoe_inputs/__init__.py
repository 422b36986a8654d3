"""Seeded synthetic inputs for the offloaded-MoE decode path.

This package only *draws inputs*: weights, a similarity table, hidden states
whose gate logits have a prescribed shape and safety margin.  It contains no
routing, substitution, cache or FFN code; both the CPU oracle and the HIP
library consume what it produces and neither is imported from here.
"""
from .shapes import MoEShape, SHAPES, shape_by_name
from .generate import Workload, make_workload, as_numpy, logit_margin_ok, chain_next_input

__all__ = [
    "MoEShape", "SHAPES", "shape_by_name",
    "Workload", "make_workload", "as_numpy", "logit_margin_ok", "chain_next_input",
]
