"""Seeded synthetic clustered-KV-cache inputs for the Double-P decode step.

This package only *draws inputs* (cluster sizes, keys, values, queries, the
per-cluster means that the prefill stage would have stored).  It contains none
of the decode method's arithmetic (no logits, softmax, top-p or attention) and
is the only module shared by the CPU oracle's tests and the HIP path's tests.
"""
from .synth import (  # noqa: F401
    ClusteredCache,
    CONFIGS,
    make_config,
    make_cache,
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    pin_sink_and_window,
    TokenOrderInput,
    token_order_input,
    CLUSTER_PINNED,
)
