"""CPU fp64 oracle for TokenRing's per-device compute path (test infrastructure only).

Nothing in the product path imports this package: only ``tests/``, the smoke check and
the benchmark's CPU-baseline leg do.  It shares no code with the HIP kernels.
"""
from .tokenring_oracle import (  # noqa: F401
    attention_block,
    attention_full,
    attention_rows,
    hybrid_order,
    merge_nary,
    merge_pair,
    merge_pair_sigmoid_form,
    ring_attention,
    ring_attention_order,
    ring_schedule,
    softmax_weights,
    zigzag_order,
    zigzag_segments,
    zigzag_steps,
)
