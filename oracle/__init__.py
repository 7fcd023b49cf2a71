"""Plain fp64 CPU oracle for the SEKA / AdaSEKA prefill hot path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this package:
it exists so that tests, the smoke check and the benchmark's CPU-baseline leg
can compare the HIP kernels with a slow, obviously correct implementation that
was written from the paper alone and shares no code with the GPU path.
"""
from .seka_oracle import (  # noqa: F401
    projector,
    blended_projector,
    edit_keys,
    causal_attention,
    steered_attention,
    attention_rows,
    route_softmax_cos,
    route_eq6,
    mean_group_query,
)
