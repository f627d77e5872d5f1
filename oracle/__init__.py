"""CPU oracle for the MoE-FFN layer.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path (the HIP library or its Python binding) may import
this package; only tests, the smoke check and the benchmark's CPU-baseline leg
use it.  It shares no code with the HIP path.
"""
from .moe_ffn_oracle import (  # noqa: F401
    backward,
    forward,
    local_permutation,
    route,
    swiglu,
    swiglu_add,
)
