"""MI355X-native (gfx950) TokenRing per-device compute path: block attention, lse merge, ring schedule.

Thin Python names over the C ABI in include/tokenring.h.  The first use of any name
loads libtokenring.so and raises ImportError if it has not been built (there is no
fallback path); `python -m paper_2412_20501_amd.build` compiles it.
"""
_EXPORTS = (
    "LIB_PATH", "TR_BF16", "TR_F32", "TR_MASK_CAUSAL_DIAG", "TR_MASK_NONE",
    "TR_SCHED_HYBRID", "TR_SCHED_RING_ATTENTION", "TR_SCHED_TOKENRING", "TR_SCHED_ZIGZAG", "TokenRingError", "TrTensor",
    "desc", "raw_lib", "tr_block_attn", "tr_block_attn_causal_at", "tr_block_attn_merge", "tr_merge", "tr_merge_n", "tr_ring_attn",
    "tr_ring_attn_blocks", "tr_ring_attn_noalloc", "tr_ring_attn_blocks_workspace_bytes", "tr_ring_attn_sched", "tr_ring_attn_workspace_bytes", "tr_schedule_steps", "tr_time_next_kernel", "tr_version",
)
__all__ = list(_EXPORTS)


def __getattr__(name):
    if name in _EXPORTS:
        from . import _binding
        return getattr(_binding, name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")
