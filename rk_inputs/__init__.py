"""Seeded synthetic inputs for the RotateK hot path.

This module only draws random numbers and rounds them to the storage dtype.
It contains none of the method's arithmetic (no covariance, rotation,
projection or attention) and is the single piece of code that both the CPU
oracle's tests and the HIP path's tests consume.

Recipe (stands in for post-RoPE visual Keys of a VLM layer, which the paper
describes as low-dimensional with a few large-magnitude outlier channels,
Sec. 3 / Fig. 2): per (layer, batch item, KV head)

    K = A @ Bm + noise * E,  A[L, rho], Bm[rho, d], E[L, d] i.i.d. N(0, 1)

then `n_outlier` distinct channels are scaled by `outlier_scale`, an optional
per-channel constant `mean_shift` is added on those outlier channels, and the
result is rounded once to the storage dtype.  Values, queries and appended
rows are N(0, 1).
"""
from .generator import (  # noqa: F401
    CONFIGS,
    HeadSpec,
    bf16_round,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    stream,
    make_keys,
    make_normal,
    make_layer,
    ragged_lengths,
    token_keep_lists,
)
