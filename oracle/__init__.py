"""fp64 CPU oracle for fused multi-head attention (test infrastructure only).

Nothing in the product package imports this; it is loaded by the tests, by the
smoke check and by the benchmark's cpu_baseline leg.
"""
from .mha_oracle import (  # noqa: F401
    OracleLib,
    build,
    compile_source,
    default,
    dropout_mask,
    mha_bwd,
    mha_fwd,
    num_threads,
    philox4x32_10,
)
