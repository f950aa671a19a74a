"""Seeded synthetic inputs for the CoCoA round (shared by the CPU oracle and the GPU path).

This package holds input generation only: data matrices, labels, chunk boundaries,
solver schedules and coordinate permutations.  It contains none of the method's
arithmetic (no dual steps, no aggregation, no gap, no assignment policy) and imports
neither the oracle nor the GPU library.
"""
from .configs import CONFIGS, get_config          # noqa: F401
from .generate import Problem, make_problem        # noqa: F401
from .permutations import chunk_draws, solver_permutation, round_permutations  # noqa: F401
