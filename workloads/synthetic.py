"""Seeded input generators and the table of workload shapes.

The paper evaluates attention at the LLaMA2-7B head shape (head dim 128, 32 heads;
Sec. 4.1) on synthetic-length sequences, so random Q/K/V of that shape *are* the
workload.  Everything here is drawn on the host from numpy's PCG64 with a fixed seed,
rounded to bf16 with round-to-nearest-even, and handed out as raw bf16 bit patterns
(uint16) so that the fp64 oracle and the GPU kernels see identical input values.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

__all__ = [
    "AttnConfig", "MergeConfig", "CONFIGS", "f32_to_bf16_bits", "bf16_bits_to_f32",
    "bf16_bits_to_f64", "make_qkv_bits", "make_merge_partials", "sample_rows",
]


@dataclass(frozen=True)
class AttnConfig:
    """One attention workload: [B, Hq, S, D] queries against [B, Hkv, S, D] keys/values."""
    name: str
    B: int
    Hq: int
    Hkv: int
    S: int          # total sequence length (for a single block step: the chunk length)
    D: int
    n_chunks: int   # chunks the ring schedule splits S into (1 = a single block step)
    causal: bool
    std: float
    seed: int
    profile: str = "normal"   # "normal": Q, K, V ~ N(0, std^2); "wide": Q and K ~ N(0, (3 std)^2); "ramp": see make_qkv_bits

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.D))

    @property
    def chunk(self) -> int:
        return self.S // self.n_chunks


@dataclass(frozen=True)
class MergeConfig:
    """Merge-only workload: n_partials fp32 partial outputs [B, H, S, D] with fp32 lse [B, H, S]."""
    name: str
    B: int
    H: int
    S: int
    D: int
    n_partials: int
    lse_lo: float
    lse_hi: float
    seed: int


CONFIGS = {
    # small non-causal case, 4 chunks of 64: 16 block steps + merges (the 4-device DiT walk-through shape)
    "cfg1_small": AttnConfig("cfg1_small", 1, 2, 2, 256, 64, 4, False, 1.0, 20502),
    # one block step, Q chunk 4096 x KV chunk 4096, 32 heads, D 128 (non-causal and diagonal-causal)
    "cfg2_block": AttnConfig("cfg2_block", 1, 32, 32, 4096, 128, 1, False, 1.0, 20503),
    "cfg2_block_diag": AttnConfig("cfg2_block_diag", 1, 32, 32, 4096, 128, 1, True, 1.0, 20503),
    # causal ring schedule, seq 32768 as 8 chunks of 4096: 36 steps
    "cfg3_ring": AttnConfig("cfg3_ring", 1, 32, 32, 32768, 128, 8, True, 1.0, 20504),
    # merge-only bandwidth test
    "cfg4_merge": MergeConfig("cfg4_merge", 1, 32, 32768, 128, 8, -5.0, 15.0, 20505),
    # GQA long context, 32 query heads / 8 KV heads, seq 131072 as 16 chunks of 8192: 136 steps
    "cfg5_gqa": AttnConfig("cfg5_gqa", 1, 32, 8, 131072, 128, 16, True, 0.5, 20506),
    # the block step on score distributions that are not N(0,1)-like: scores with a standard deviation of about 9
    # (Q and K three times wider), and scores that rise slowly and steadily along the keys (about +41 over the chunk)
    "cfg2_block_wide": AttnConfig("cfg2_block_wide", 1, 32, 32, 4096, 128, 1, False, 1.0, 20508, "wide"),
    "cfg2_block_ramp": AttnConfig("cfg2_block_ramp", 1, 32, 32, 4096, 128, 1, False, 1.0, 20509, "ramp"),
    # diffusion-transformer shaped: long non-causal sequence, head dim 64, batch 2, four devices (Sec. 3.3.1)
    "dit_ring": AttnConfig("dit_ring", 2, 24, 24, 16384, 64, 4, False, 1.0, 20507),
}


RAMP_STEP = 0.01   # rise of the scaled score per key in the "ramp" profile


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bf16 (round to nearest, ties to even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounding_bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + rounding_bias) >> 16).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float64."""
    return bf16_bits_to_f32(bits).astype(np.float64)


def _normal_bits(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    """N(0, std^2) draws rounded to bf16, generated one head at a time to bound host memory."""
    out = np.empty(shape, dtype=np.uint16)
    flat = out.reshape(-1, shape[-2], shape[-1])
    for i in range(flat.shape[0]):
        x = rng.standard_normal(flat.shape[1:], dtype=np.float32)
        if std != 1.0:
            x *= np.float32(std)
        flat[i] = f32_to_bf16_bits(x)
    return out


def make_qkv_bits(cfg: AttnConfig):
    """Q [B,Hq,S,D], K and V [B,Hkv,S,D] as bf16 bit patterns, drawn in that order from one stream."""
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    qk_std = cfg.std * (3.0 if cfg.profile == "wide" else 1.0)
    q = _normal_bits(rng, (cfg.B, cfg.Hq, cfg.S, cfg.D), qk_std)
    k = _normal_bits(rng, (cfg.B, cfg.Hkv, cfg.S, cfg.D), qk_std)
    v = _normal_bits(rng, (cfg.B, cfg.Hkv, cfg.S, cfg.D), cfg.std)
    if cfg.profile == "ramp":
        # component 0 of every query is 1 and of key c is c * RAMP_STEP / scale, so the scaled score of key c
        # carries a term c * RAMP_STEP on top of the N(0,1)-like rest: a slow, steady rise along the keys
        q[..., 0] = f32_to_bf16_bits(np.ones(1, dtype=np.float32))[0]
        ramp = (np.arange(cfg.S, dtype=np.float32) * np.float32(RAMP_STEP / cfg.scale))
        k[..., 0] = f32_to_bf16_bits(ramp)[None, None, :]
    elif cfg.profile not in ("normal", "wide"):
        raise ValueError(f"unknown profile {cfg.profile!r}")
    return q, k, v


def make_merge_partials(cfg: MergeConfig, S: int | None = None):
    """n_partials x (out fp32 [B,H,S,D] ~ N(0,1), lse fp32 [B,H,S] ~ U(lse_lo, lse_hi)).

    ``S`` overrides the sequence length (the down-scaled case the oracle checks in full).
    """
    S = cfg.S if S is None else S
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    outs, lses = [], []
    for _ in range(cfg.n_partials):
        outs.append(rng.standard_normal((cfg.B, cfg.H, S, cfg.D), dtype=np.float32))
        u = rng.random((cfg.B, cfg.H, S), dtype=np.float32)
        lses.append((np.float32(cfg.lse_lo) + u * np.float32(cfg.lse_hi - cfg.lse_lo)).astype(np.float32))
    return outs, lses


def sample_rows(S: int, chunk: int, n_random: int, seed: int) -> np.ndarray:
    """Query positions to check at full size: the first rows, every chunk boundary -1/0/+1,
    the last rows, plus ``n_random`` seeded positions.  Sorted, unique."""
    rows = {0, 1, 2, S - 2, S - 1}
    for b in range(chunk, S, chunk):
        rows.update((b - 1, b, b + 1))
    rng = np.random.Generator(np.random.PCG64(seed))
    rows.update(int(r) for r in rng.integers(0, S, size=n_random))
    return np.array(sorted(r for r in rows if 0 <= r < S), dtype=np.int64)
