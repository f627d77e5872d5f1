"""Seeded synthetic workloads for the Dispatch-to-Combine MoE-FFN layer.

This module only *draws inputs*: shapes, seeds, value distributions and the
bf16 rounding of stored values.  It holds none of the layer's arithmetic, so
both the CPU oracle's tests and the HIP path's tests can feed from it without
sharing any code of the method itself.

The shapes follow the module evaluated in the paper's Section 5.2 (hidden
7168, intermediate 2048, top-8, sequence 4096 x microbatch 2) plus smaller
parity cases.  No dataset is involved; routing logits are Gaussian, optionally
with a Zipf-like per-expert bias to imitate skewed ("natural") routing.
"""
from .configs import (  # noqa: F401
    CONFIGS,
    MoeConfig,
    bf16_round,
    expert_bias,
    make_inputs,
    make_microbench_inputs,
    realised_local_counts,
)
