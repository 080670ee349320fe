"""Seeded synthetic inputs for the aggregation path (shared by tests, smoke and bench).

Holds no part of the method under test: only the generators of the stacked worker returns
(honest file gradients and the attack payloads of Sec. 6.1) and the table of workloads.
"""
from .configs import CONFIGS, Config  # noqa: F401
from .gradients import (  # noqa: F401
    alie_vector,
    build_copies,
    honest_gradients,
    padded_ld,
)
