"""CPU oracle for the MoE layer with dynamic expert duplication (MoE-GPS setting).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, obviously-correct CPU
statement of what the GPU library computes, written from the paper.  It shares
no code with the HIP path and must never be imported by it; only the tests, the
smoke check and the benchmark's CPU-baseline leg call it.

Every function cites the passage of the paper it follows.  Where the paper is
silent the reading taken is stated in the function's docstring.
"""
from .routing import route_topk
from .histogram import histogram, skewness, dist_error_rate
from .plan import plan_duplicates, home_slot, Plan
from .permute import permute, dispatch_segments
from .ffn import grouped_ffn, ffn_rows
from .combine import combine
from .layer import moe_layer

__all__ = [
    "route_topk", "histogram", "skewness", "dist_error_rate", "plan_duplicates", "home_slot",
    "Plan", "permute", "dispatch_segments", "grouped_ffn", "ffn_rows", "combine", "moe_layer",
]
