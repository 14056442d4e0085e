"""Helpers shared by the GPU parity tests: host bits -> device tensors, oracle-side views."""
import numpy as np
import torch

import oracle
import workloads as wl


def bits_to_dev(bits: np.ndarray) -> torch.Tensor:
    """bf16 bit patterns (uint16 numpy) -> bf16 torch tensor on cuda:0 with the same bits."""
    return torch.from_numpy(bits.view(np.int16)).to("cuda").view(torch.bfloat16)


def rand_bits(shape, seed, std=1.0):
    rng = np.random.Generator(np.random.PCG64(seed))
    return wl.f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32) * np.float32(std))


def f64(bits):
    return wl.bf16_bits_to_f64(bits)


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def max_abs(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    both_ninf = np.isneginf(a) & np.isneginf(b)
    d = np.abs(np.where(both_ninf, 0.0, a) - np.where(both_ninf, 0.0, b))
    return float(np.max(d)) if d.size else 0.0


def check_rows(cfg, out, lse, qb, kb, vb, n_random, heads=None):
    """Compare sampled rows of every head against exact oracle rows."""
    rows = wl.sample_rows(cfg.S, cfg.chunk, n_random, seed=cfg.seed + 1)
    G = cfg.Hq // cfg.Hkv
    worst_o = worst_l = 0.0
    ridx = torch.from_numpy(rows).to("cuda")
    for h in (range(cfg.Hq) if heads is None else heads):
        g = h // G
        ref_o, ref_l = oracle.attention_rows(f64(qb[0, h][rows]), rows, f64(kb[0, g]), f64(vb[0, g]), cfg.scale, cfg.causal)
        worst_o = max(worst_o, max_abs(to_np(out[0, h][ridx]), ref_o))
        worst_l = max(worst_l, max_abs(to_np(lse[0, h][ridx]), ref_l))
    return worst_o, worst_l, len(rows)
