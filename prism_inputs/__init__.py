"""Seeded synthetic workloads for one edge server's MoE layer (Prism, Sec. III-A).

This module only *draws inputs*: tokens, router / expert weights, the Zipf
popularity bias and the per-server placement mask.  It holds none of the
method's arithmetic (no routing, no FFN, no combine), so both the CPU oracle's
tests and the HIP path's tests can consume it without sharing code.

The paper measures on trained Mixtral-8x7B / DeepSeek-V2-Lite weights and
public prompt sets (Sec. IV, "Models and datasets"); neither is available
here, so these tensors stand in for them.  They keep the layer shapes of the
two model families and the two workload properties the method depends on:
skewed, task dependent expert popularity (Sec. II-B, Fig. 2) and its drift
over time (Sec. III-C "Expert Migration", Fig. 6).
"""
from .generate import (  # noqa: F401
    CONFIGS,
    LayerConfig,
    LayerInputs,
    bf16_bits_to_f32,
    f32_to_bf16_bits,
    make_inputs,
    make_config,
    zipf_bias,
    top_popular_mask,
    random_mask,
)
