"""Seeded synthetic inputs (sparse matrices, embedding tables) for the iALS path.

This package holds input generation only: none of the method's arithmetic lives
here.  Both the CPU oracle's tests and the GPU path's tests draw their inputs
from it, so the two sides always see identical arrays.
"""
from .matrices import (  # noqa: F401
    CONFIGS,
    SparseProblem,
    csr_from_edges,
    extract_rows,
    hash_u64,
    holdout_split,
    init_table,
    make_problem,
    transpose_csr,
    uniform01,
)
