"""CPU oracle for the relay-race ranking path.  TEST INFRASTRUCTURE ONLY.

Nothing under this package is part of the product: only the tests, the smoke
check and the benchmark's cpu_baseline leg may import it.  It shares no code
with the HIP path and never imports it.
"""
from .relaygr_oracle import (  # noqa: F401
    layer_norm,
    silu,
    visibility_mask,
    backbone_layer,
    full_recompute,
    prefix_kv,
    rank_with_kv,
    score_head,
    kv_footprint_bytes,
)
from .brute_force import brute_force_scores  # noqa: F401
