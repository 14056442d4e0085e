"""GPU parity of tr_ring_attn (Algorithm 1's schedule on one GPU) against the fp64 oracle.

The reference is *unchunked* fp64 attention: the chunked schedule must reach it within
max-abs 1e-2 on out and 1e-3 on lse.  The large workloads are checked on a row sample
(all heads; first rows, every chunk boundary -1/0/+1, last rows, seeded random rows),
each sampled row computed exactly by the oracle.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from gpu_util import bits_to_dev, check_rows as _check_rows, f64, max_abs, rand_bits, to_np

pytestmark = pytest.mark.gpu
OUT_TOL, LSE_TOL = 1e-2, 1e-3


def _ring(lib, q, k, v, n_chunks, causal, scale=0.0, poison=True, fused=True):
    """fused=True: Update in the attention epilogue (no workspace); False: tr_block_attn + tr_merge."""
    B, Hq, S, D = q.shape
    fill = float("nan") if poison else 0.0
    out = torch.full((B, Hq, S, D), fill, dtype=torch.float32, device="cuda")
    lse = torch.full((B, Hq, S), fill, dtype=torch.float32, device="cuda")
    ws = None if fused else torch.empty(max(256, lib.tr_ring_attn_workspace_bytes(q, n_chunks)), dtype=torch.uint8, device="cuda")
    lib.tr_ring_attn(q, k, v, n_chunks, causal, out, lse, scale, ws)
    torch.cuda.synchronize()
    return out, lse


def test_ring_config1_small_noncausal_16_steps(lib):
    cfg = wl.CONFIGS["cfg1_small"]
    qb, kb, vb = wl.make_qkv_bits(cfg)
    out, lse = _ring(lib, bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb), cfg.n_chunks, cfg.causal, cfg.scale)
    ref_o, ref_l = oracle.attention_full(f64(qb), f64(kb), f64(vb), cfg.scale, causal=False)
    assert max_abs(to_np(out), ref_o) <= OUT_TOL and max_abs(to_np(lse), ref_l) <= LSE_TOL
    # the oracle's own replay of Algorithm 1 agrees with the same tolerance
    alg_o, alg_l = oracle.ring_attention(f64(qb), f64(kb), f64(vb), cfg.n_chunks, False, cfg.scale)
    assert max_abs(to_np(out), alg_o) <= OUT_TOL and max_abs(to_np(lse), alg_l) <= LSE_TOL


@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("n_chunks", [1, 2, 3, 8])
def test_ring_chunk_count_invariance(lib, n_chunks, causal, fused):
    B, Hq, Hkv, S, D = 2, 4, 2, 384, 128          # chunk of 128 / 48: several waves and a ragged tile tail
    qb, kb, vb = rand_bits((B, Hq, S, D), 21), rand_bits((B, Hkv, S, D), 22), rand_bits((B, Hkv, S, D), 23)
    out, lse = _ring(lib, bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb), n_chunks, causal, fused=fused)   # scale 0 -> 1/sqrt(D)
    ref_o, ref_l = oracle.attention_full(f64(qb), f64(kb), f64(vb), 1.0 / np.sqrt(D), causal)
    assert max_abs(to_np(out), ref_o) <= OUT_TOL and max_abs(to_np(lse), ref_l) <= LSE_TOL


def test_ring_n1_equals_single_block_step_bitwise(lib):
    qb, kb, vb = rand_bits((1, 2, 320, 128), 24), rand_bits((1, 2, 320, 128), 25), rand_bits((1, 2, 320, 128), 26)
    q, k, v = bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb)
    out, lse = _ring(lib, q, k, v, 1, True, 0.07)
    o2 = torch.empty_like(out); l2 = torch.empty_like(lse)
    lib.tr_block_attn(q, k, v, lib.TR_MASK_CAUSAL_DIAG, 0.07, o2, l2)
    torch.cuda.synchronize()
    assert torch.equal(out, o2) and torch.equal(lse, l2)


def test_fused_and_two_kernel_forms_agree(lib):
    """Same Update arithmetic in the same order: the fused epilogue and tr_block_attn + tr_merge
    differ only in how the block reaches the Update (fp32 registers vs an fp32 workspace)."""
    qb, kb, vb = rand_bits((1, 4, 1024, 128), 30), rand_bits((1, 2, 1024, 128), 31), rand_bits((1, 2, 1024, 128), 32)
    q, k, v = bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb)
    a = _ring(lib, q, k, v, 4, True, fused=True)
    b = _ring(lib, q, k, v, 4, True, fused=False)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_block_attn_merge_matches_oracle_update(lib):
    """tr_block_attn_merge on random fp32 accumulators (some rows empty) vs oracle attention + oracle Update."""
    B, Hq, Hkv, Sq, Sk, D = 1, 4, 2, 300, 200, 128
    qb, kb, vb = rand_bits((B, Hq, Sq, D), 33), rand_bits((B, Hkv, Sk, D), 34), rand_bits((B, Hkv, Sk, D), 35)
    rng = np.random.default_rng(36)
    acc_o = rng.standard_normal((B, Hq, Sq, D)).astype(np.float32)
    acc_l = rng.uniform(-5, 15, (B, Hq, Sq)).astype(np.float32)
    acc_l[0, 0, :7] = -np.inf
    acc_o[0, 0, :7] = np.nan                         # empty rows may hold garbage
    d_o, d_l = torch.from_numpy(acc_o).to("cuda"), torch.from_numpy(acc_l).to("cuda")
    lib.tr_block_attn_merge(bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb), lib.TR_MASK_NONE, 0.09, d_o, d_l)
    torch.cuda.synchronize()
    blk_o, blk_l = oracle.attention_block(f64(qb), f64(kb), f64(vb), 0.09)
    clean = acc_o.copy(); clean[0, 0, :7] = 0.0
    ref_o, ref_l = oracle.merge_pair(clean, acc_l, blk_o, blk_l)
    assert not torch.isnan(d_o).any()
    assert max_abs(to_np(d_o), ref_o) <= OUT_TOL and max_abs(to_np(d_l), ref_l) <= LSE_TOL


def test_ring_is_bitwise_reproducible(lib):
    qb, kb, vb = rand_bits((1, 4, 512, 64), 27), rand_bits((1, 4, 512, 64), 28), rand_bits((1, 4, 512, 64), 29)
    q, k, v = bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb)
    a = _ring(lib, q, k, v, 4, True)
    b = _ring(lib, q, k, v, 4, True, poison=False)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_ring_config3_causal_32k_8_chunks_sampled_rows(lib):
    cfg = wl.CONFIGS["cfg3_ring"]
    qb, kb, vb = wl.make_qkv_bits(cfg)
    out, lse = _ring(lib, bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb), cfg.n_chunks, cfg.causal, cfg.scale)
    assert not torch.isnan(out).any() and not torch.isnan(lse).any()
    worst_o, worst_l, n = _check_rows(cfg, out, lse, qb, kb, vb, n_random=256)
    print(f"cfg3: {n} rows x {cfg.Hq} heads, max|d out| {worst_o:.3e}, max|d lse| {worst_l:.3e}")
    assert worst_o <= OUT_TOL and worst_l <= LSE_TOL


def test_ring_dit_shape_noncausal_d64_sampled_rows(lib):
    """Non-causal, head dim 64, batch 2, four devices (the diffusion-transformer case study): batch 0 is checked."""
    cfg = wl.CONFIGS["dit_ring"]
    qb, kb, vb = wl.make_qkv_bits(cfg)
    out, lse = _ring(lib, bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb), cfg.n_chunks, cfg.causal, cfg.scale)
    assert not torch.isnan(out).any() and not torch.isnan(lse).any()
    worst_o, worst_l, n = _check_rows(cfg, out, lse, qb, kb, vb, n_random=64)
    print(f"dit: {n} rows x {cfg.Hq} heads, max|d out| {worst_o:.3e}, max|d lse| {worst_l:.3e}")
    assert worst_o <= OUT_TOL and worst_l <= LSE_TOL
    # second batch entry: a few heads
    rows = wl.sample_rows(cfg.S, cfg.chunk, 16, seed=cfg.seed + 2)
    ridx = torch.from_numpy(rows).to("cuda")
    for h in (0, 11, 23):
        ref_o, ref_l = oracle.attention_rows(f64(qb[1, h][rows]), rows, f64(kb[1, h]), f64(vb[1, h]), cfg.scale, False)
        assert max_abs(to_np(out[1, h][ridx]), ref_o) <= OUT_TOL and max_abs(to_np(lse[1, h][ridx]), ref_l) <= LSE_TOL


def test_ring_config5_gqa_128k_16_chunks_sampled_rows(lib):
    cfg = wl.CONFIGS["cfg5_gqa"]
    qb, kb, vb = wl.make_qkv_bits(cfg)
    out, lse = _ring(lib, bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb), cfg.n_chunks, cfg.causal, cfg.scale)
    assert not torch.isnan(lse).any()
    worst_o, worst_l, n = _check_rows(cfg, out, lse, qb, kb, vb, n_random=96)
    print(f"cfg5: {n} rows x {cfg.Hq} heads, max|d out| {worst_o:.3e}, max|d lse| {worst_l:.3e}")
    assert worst_o <= OUT_TOL and worst_l <= LSE_TOL


def test_ring_blocks_fp32_is_the_two_kernel_form_bitwise(lib):
    qb, kb, vb = rand_bits((1, 4, 768, 128), 50), rand_bits((1, 2, 768, 128), 51), rand_bits((1, 2, 768, 128), 52)
    q, k, v = bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb)
    a = _ring(lib, q, k, v, 3, True, fused=False)
    out = torch.full_like(a[0], float("nan")); lse = torch.full_like(a[1], float("nan"))
    ws = torch.empty(lib.tr_ring_attn_blocks_workspace_bytes(q, 3, lib.TR_F32), dtype=torch.uint8, device="cuda")
    assert ws.numel() == lib.tr_ring_attn_workspace_bytes(q, 3)
    lib.tr_ring_attn_blocks(q, k, v, 3, True, out, lse, lib.TR_F32, ws)
    torch.cuda.synchronize()
    assert torch.equal(out, a[0]) and torch.equal(lse, a[1])


@pytest.mark.parametrize("causal", [False, True])
def test_ring_blocks_bf16_transport(lib, causal):
    """block_out stored as bf16 between Attention and Update: every merged block carries one bf16 rounding,
    i.e. at most 2^-8 of the largest block value on top of the kernel's own 1e-2; lse is untouched by it."""
    B, Hq, Hkv, S, D, n = 1, 4, 2, 1024, 128, 4
    qb, kb, vb = rand_bits((B, Hq, S, D), 53), rand_bits((B, Hkv, S, D), 54), rand_bits((B, Hkv, S, D), 55)
    q, k, v = bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb)
    out = torch.full((B, Hq, S, D), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((B, Hq, S), float("nan"), dtype=torch.float32, device="cuda")
    nbytes = lib.tr_ring_attn_blocks_workspace_bytes(q, n, lib.TR_BF16)
    assert nbytes == Hq * (S // n) * D * 2 + Hq * (S // n) * 4
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    lib.tr_ring_attn_blocks(q, k, v, n, causal, out, lse, lib.TR_BF16, ws)
    torch.cuda.synchronize()
    ref_o, ref_l = oracle.attention_full(f64(qb), f64(kb), f64(vb), 1.0 / np.sqrt(D), causal)
    vmax = float(np.abs(f64(vb)).max())
    d_o, d_l = max_abs(to_np(out), ref_o), max_abs(to_np(lse), ref_l)
    print(f"bf16 transport, causal={causal}: max|d out| {d_o:.3e} (bound {OUT_TOL + vmax * 2.0 ** -8:.3e}), max|d lse| {d_l:.3e}")
    assert d_o <= OUT_TOL + vmax * 2.0 ** -8 and d_l <= LSE_TOL
    # and the same order of Updates with the oracle's blocks rounded to bf16 on the way (first block of a chunk is not)
    C = S // n
    o_ref = np.zeros((B, Hq, S, D)); l_ref = np.full((B, Hq, S), -np.inf)
    seen = set()
    for _, j, c in oracle.ring_schedule(n, causal):
        qs, ks = slice(c * C, (c + 1) * C), slice(j * C, (j + 1) * C)
        bo, bl = oracle.attention_block(f64(qb)[:, :, qs], f64(kb)[:, :, ks], f64(vb)[:, :, ks], 1.0 / np.sqrt(D),
                                        causal_diag=causal, q_offset=c * C, k_offset=j * C)
        if c in seen:
            bo = wl.bf16_bits_to_f64(wl.f32_to_bf16_bits(bo.astype(np.float32)))
        seen.add(c)
        o_ref[:, :, qs], l_ref[:, :, qs] = oracle.merge_pair(o_ref[:, :, qs], l_ref[:, :, qs], bo, bl)
    assert max_abs(to_np(out), o_ref) <= OUT_TOL + vmax * 2.0 ** -8 and max_abs(to_np(lse), l_ref) <= LSE_TOL


def test_ring_config3_bf16_transport_sampled_rows(lib):
    """cfg3 in the two-kernel form with bf16 block_out between Attention and Update (one bf16 rounding per merged block)."""
    cfg = wl.CONFIGS["cfg3_ring"]
    qb, kb, vb = wl.make_qkv_bits(cfg)
    q, k, v = bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb)
    out = torch.full((cfg.B, cfg.Hq, cfg.S, cfg.D), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((cfg.B, cfg.Hq, cfg.S), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(lib.tr_ring_attn_blocks_workspace_bytes(q, cfg.n_chunks, lib.TR_BF16), dtype=torch.uint8, device="cuda")
    lib.tr_ring_attn_blocks(q, k, v, cfg.n_chunks, True, out, lse, lib.TR_BF16, ws, cfg.scale)
    torch.cuda.synchronize()
    assert not torch.isnan(out).any() and not torch.isnan(lse).any()
    worst_o, worst_l, n = _check_rows(cfg, out, lse, qb, kb, vb, n_random=128)
    vmax = float(np.abs(f64(vb)).max())
    print(f"cfg3 bf16 transport: {n} rows x {cfg.Hq} heads, max|d out| {worst_o:.3e} (bound {OUT_TOL + vmax * 2.0 ** -8:.3e}), max|d lse| {worst_l:.3e}")
    assert worst_o <= OUT_TOL + vmax * 2.0 ** -8 and worst_l <= LSE_TOL
