"""Seeded synthetic inputs for the active-weight decode path.

This module only draws random numbers and shapes them into the tensors the
workloads need (weights, activations, KV caches, norm gains).  It holds none
of the method's arithmetic: no selection, no masking, no GEMV, no quantiser.
Both the CPU oracle's tests and the HIP path's tests/bench feed from here, so
the two sides always see the same fp16 bits.

Recipe (stand-in for the LLaMA-family checkpoints and text corpora the paper
measures on, which are not available offline):
  * weights  W[out][in] ~ N(0, 0.02), rounded to fp16;
  * activations x_j = fp16(Laplace(0,1) * s_j) with a per-channel log-normal
    scale s_j = exp(0.5 z_j), z_j ~ N(0,1), drawn once per model and shared by
    every token, and max(1, round(0.001 n)) outlier channels whose scale is
    multiplied by 20;
  * norm gains g = 1 + N(0, 0.02) in fp16; KV cache entries ~ N(0,1) in fp16.
Every tensor has its own child stream keyed by (seed, tag...), so generation
order never matters.
"""
from .generators import (  # noqa: F401
    MODEL_SHAPES,
    ModelShape,
    activation,
    channel_scales,
    device_kv_cache,
    device_layer_weights,
    device_moe_layer_weights,
    kv_cache,
    layer_weights,
    moe_layer_weights,
    norm_gain,
    rng_for,
    weight_matrix,
)
