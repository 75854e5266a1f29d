"""Fused multi-head attention (forward + backward) for MI355X, behind a C ABI.

``binding`` marshals torch device tensors into ``libspark_mha.so``;
``synth`` generates the seeded synthetic workloads; ``build`` compiles the library.
"""
from .binding import (  # noqa: F401
    EXPORTS,
    HipEvents,
    SparkError,
    Strides,
    load_library,
    spark_dropout_mask,
    spark_dropout_threshold,
    spark_layout_probe,
    spark_mha_bwd,
    spark_mha_bwd_atomic,
    spark_mha_bwd_atomic_workspace_bytes,
    spark_mha_bwd_static,
    spark_mha_bwd_static_max_rows,
    spark_mha_bwd_workspace_bytes,
    spark_mha_cross_bwd,
    spark_mha_cross_bwd_workspace_bytes,
    spark_mha_cross_fwd,
    spark_mha_dropout_bwd,
    spark_mha_dropout_fwd,
    spark_mha_fwd,
    spark_mha_strided_bwd,
    spark_mha_strided_fwd,
    status_str,
)
