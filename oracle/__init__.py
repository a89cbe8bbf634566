"""fp64 CPU oracle of the MoE layer -- TEST INFRASTRUCTURE ONLY.

Nothing on the product path may import this package; it shares no code with the
HIP library.  See moe_oracle.c for what it computes and how it is pinned.
"""
from .moe_oracle import (  # noqa: F401
    OracleProblem,
    gate,
    plan,
    layer,
    num_threads,
    bf16_bits_to_f64,
)
