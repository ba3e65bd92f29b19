"""Seeded synthetic inputs for the batched verification pass.

This package only draws random numbers and moves bytes around (shapes, paging,
dtype rounding and widening).  It holds none of the method's arithmetic, so the
CPU oracle and the HIP path can both be fed from it without sharing code.
"""
from .synth import (  # noqa: F401
    ModelCfg,
    Workload,
    Weights,
    KVCache,
    Batch,
    OracleModelView,
    OracleKVView,
    config,
    tiny_workload,
    make_weights,
    make_batch,
    make_seeded_kv,
    make_prefix_ids,
    pages_from_dense,
    draw_verdict_ids,
    torch_dtype,
    DRAFT_SHAPE,
    TARGET_SHAPE,
)
