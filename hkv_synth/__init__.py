"""Seeded synthetic inputs for the HybridKV hot path.

This package only draws random tensors and lays out tokens, head types and
budgets.  It holds none of the method's arithmetic (no scoring, selection,
chunk summaries or attention): both the CPU oracle's tests and the HIP path's
tests/bench take their inputs from here, and nothing else is shared between
the two.
"""
from .workloads import (  # noqa: F401
    make_prompt_queries,
    CONFIGS,
    Workload,
    bf16_round,
    make_workload,
    token_layout,
)
