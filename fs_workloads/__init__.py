"""Seeded synthetic input generators shared by the CPU oracle tests and the HIP path.

Only inputs are produced here (jagged ID batches, per-occurrence gradients, the
table-initialisation rule).  None of the method's arithmetic (gather, dedup,
collision split, segment reduce, Adagrad) lives in this package, and it imports
neither the oracle nor the HIP binding.
"""
from .generators import (  # noqa: F401
    CONFIGS,
    TableSpec,
    WorkloadConfig,
    Iteration,
    bounded_zipf_ranks,
    rank_to_row,
    powerlaw_lengths,
    make_iterations,
    hash_init_rows,
    mix32,
    compact_rows,
)
