"""fp64 CPU oracle for the VLA forward recurrence -- test infrastructure only.

Nothing in the product package imports this.  Allowed callers: tests/, the
smoke check and the benchmark's cpu_baseline leg.
"""
from .oracle_lib import (  # noqa: F401
    TRACE_WIDTH,
    forward,
    linear_attention,
    num_threads,
    load,
)
