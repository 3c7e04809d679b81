"""fp64 CPU oracle for partitioned decode attention -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this package.
The product path (the HIP library and its binding) never does.
"""
from .oracle import (  # noqa: F401
    attn_concat,
    attn_full,
    attn_gather,
    attn_logits,
    attn_merge,
    attn_partial,
    attn_select,
    attn_topk,
    build,
    max_threads,
)
