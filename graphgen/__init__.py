"""Seeded synthetic graph generators shared by the tests, the oracle drivers and
the benchmark.

This module only produces *inputs* (edge lists, CSR arrays, train/test edge
splits).  It holds none of the embedding method's arithmetic: no sampling rule,
no update rule, no coarsening.  Everything is written with torch tensor ops so
the same code runs on the CPU (small graphs in the unit tests) and on a GPU
(the 2^24-vertex benchmark graph is generated in HBM in a few seconds).

The graphs stand in for the real-world social / web graphs the paper evaluates
on (its dataset table): heavy-tailed degree distributions with mean degree in
the 3..40 range.
"""
from .generators import (
    er_gnm,
    rmat,
    chung_lu,
    holdout_split,
    to_csr,
    two_cliques,
    CSR,
)

__all__ = [
    "er_gnm",
    "rmat",
    "chung_lu",
    "holdout_split",
    "to_csr",
    "two_cliques",
    "CSR",
]
