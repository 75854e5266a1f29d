"""fp64 CPU oracle for fused multi-head attention (test infrastructure only).

Nothing in the product package imports this; it is loaded by the tests, by the
smoke check and by the benchmark's cpu_baseline leg.
"""
from .mha_oracle import (  # noqa: F401
    build,
    num_threads,
    mha_fwd,
    mha_bwd,
)
