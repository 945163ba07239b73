"""Seeded synthetic inputs for a Parameter-Server ranking-model iteration.

This package only *draws inputs* (ids, bag lengths, dense features, labels,
initial parameters).  It holds none of the arithmetic of the training step
itself and is the one module both the CPU oracle's tests and the GPU path's
tests are allowed to share.
"""
from .gen import (  # noqa: F401
    SEED0,
    Batch,
    RankingConfig,
    DenseConfig,
    CONFIGS,
    DENSE_CONFIG,
    fmix32,
    table_values,
    make_tables,
    make_mlp_params,
    make_batch,
    make_dense_problem,
    scaled,
    table_rows_f32,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    param_layout,
    split_params,
    batch_from_bags,
    shard_slices,
)
