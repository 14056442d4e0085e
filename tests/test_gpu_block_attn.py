"""GPU parity of tr_block_attn / tr_block_attn_causal_at against the fp64 oracle.

Tolerances (bf16 inputs, fp32 accumulation, probabilities rounded to bf16 before PV):
max-abs 1e-2 on block_out, 1e-3 on the fp32 block_lse.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from gpu_util import bits_to_dev, f64, max_abs, rand_bits, to_np

pytestmark = pytest.mark.gpu
OUT_TOL, LSE_TOL = 1e-2, 1e-3


def _run_block(lib, qb, kb, vb, scale, mask, out_dtype, causal_at=None):
    q, k, v = bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb)
    B, Hq, Sq, D = q.shape
    out = torch.full((B, Hq, Sq, D), float("nan"), dtype=out_dtype, device="cuda")
    lse = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device="cuda")
    if causal_at is None:
        lib.tr_block_attn(q, k, v, mask, scale, out, lse)
    else:
        lib.tr_block_attn_causal_at(q, k, v, causal_at[0], causal_at[1], scale, out, lse)
    torch.cuda.synchronize()
    return to_np(out), to_np(lse)


SHAPES = [
    # B, Hq, Hkv, Sq, Sk, D
    (1, 2, 2, 64, 64, 64),
    (1, 2, 1, 256, 256, 128),
    (2, 4, 2, 300, 300, 128),     # ragged tail in both Sq and Sk, GQA, batch 2
    (1, 1, 1, 1, 1, 128),
    (1, 3, 3, 33, 500, 64),       # Sq < one wave, several K/V tiles + tail
    (1, 2, 2, 513, 65, 128),      # three query tiles (last nearly empty), key tail of 1
    (1, 8, 8, 512, 1024, 128),    # exercises the XCD-aware block mapping
    (1, 24, 8, 300, 300, 128),    # XCD-aware mapping with three query heads per K/V head (not a power of two)
    (2, 16, 8, 260, 260, 64),     # XCD-aware mapping with batch 2 (16 K/V heads over 8 XCDs), head dim 64
]


@pytest.mark.parametrize("out_dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("shape", SHAPES)
def test_block_attn_no_mask(lib, shape, out_dtype):
    B, Hq, Hkv, Sq, Sk, D = shape
    qb, kb, vb = rand_bits((B, Hq, Sq, D), 1), rand_bits((B, Hkv, Sk, D), 2), rand_bits((B, Hkv, Sk, D), 3)
    scale = 1.0 / np.sqrt(D)
    out, lse = _run_block(lib, qb, kb, vb, scale, lib.TR_MASK_NONE, out_dtype)
    ref_o, ref_l = oracle.attention_block(f64(qb), f64(kb), f64(vb), scale)
    assert max_abs(out, ref_o) <= OUT_TOL and max_abs(lse, ref_l) <= LSE_TOL


def test_block_attn_more_heads_than_the_head_major_grid_holds(lib):
    """B * Hq / 8 beyond 65535 (the y extent of a grid): the launch keeps batch*head in x.  Sampled heads against the oracle."""
    B, H, Sq, Sk, D = 1, 8 * 65537, 2, 3, 64
    g = torch.Generator(device="cuda").manual_seed(77)
    q = torch.randn((B, H, Sq, D), device="cuda", generator=g).bfloat16()
    k = torch.randn((B, H, Sk, D), device="cuda", generator=g).bfloat16()
    v = torch.randn((B, H, Sk, D), device="cuda", generator=g).bfloat16()
    out = torch.full((B, H, Sq, D), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((B, H, Sq), float("nan"), dtype=torch.float32, device="cuda")
    lib.tr_block_attn(q, k, v, lib.TR_MASK_NONE, 0.125, out, lse)
    torch.cuda.synchronize()
    assert not torch.isnan(out).any() and not torch.isnan(lse).any()
    heads = sorted({0, 1, 7, 8, 9, 65535, 65536, 65537, 8 * 65535, 8 * 65536 - 1, 8 * 65536, H - 9, H - 8, H - 1} | set(range(100000, H, 77773)))
    hs = torch.tensor(heads, device="cuda")
    sel = lambda t: t.index_select(1, hs).float().cpu().numpy().astype(np.float64)
    ref_o, ref_l = oracle.attention_block(sel(q), sel(k), sel(v), 0.125)
    assert max_abs(sel(out), ref_o) <= OUT_TOL and max_abs(lse.index_select(1, hs).cpu().numpy().astype(np.float64), ref_l) <= LSE_TOL


@pytest.mark.parametrize("shape", [s for s in SHAPES if s[3] == s[4]] + [(1, 2, 2, 1000, 1000, 128)])
def test_block_attn_causal_diag(lib, shape):
    B, Hq, Hkv, Sq, Sk, D = shape
    qb, kb, vb = rand_bits((B, Hq, Sq, D), 4), rand_bits((B, Hkv, Sk, D), 5), rand_bits((B, Hkv, Sk, D), 6)
    scale = 1.0 / np.sqrt(D)
    out, lse = _run_block(lib, qb, kb, vb, scale, lib.TR_MASK_CAUSAL_DIAG, torch.float32)
    ref_o, ref_l = oracle.attention_block(f64(qb), f64(kb), f64(vb), scale, causal_diag=True)
    assert max_abs(out, ref_o) <= OUT_TOL and max_abs(lse, ref_l) <= LSE_TOL
    # row 0 sees only key 0: out = v0 up to fp32 rounding of the softmax shift
    assert max_abs(out[:, :, 0], np.repeat(f64(vb), Hq // Hkv, axis=1)[:, :, 0]) <= 2e-6


@pytest.mark.parametrize("pos", [(0, 0), (256, 0), (0, 256), (100, 37), (37, 100), (64, 1000), (5, 200)])
def test_block_attn_causal_at_offsets(lib, pos):
    """Causal rule at arbitrary chunk positions, including rows that see no key at all."""
    B, Hq, Hkv, Sq, Sk, D = 1, 2, 1, 200, 160, 128
    qb, kb, vb = rand_bits((B, Hq, Sq, D), 7), rand_bits((B, Hkv, Sk, D), 8), rand_bits((B, Hkv, Sk, D), 9)
    scale = 0.11
    out, lse = _run_block(lib, qb, kb, vb, scale, None, torch.float32, causal_at=pos)
    ref_o, ref_l = oracle.attention_block(f64(qb), f64(kb), f64(vb), scale, causal_diag=True, q_offset=pos[0], k_offset=pos[1])
    assert np.array_equal(np.isneginf(lse), np.isneginf(ref_l))
    assert max_abs(out, ref_o) <= OUT_TOL and max_abs(lse, ref_l) <= LSE_TOL
    assert not np.isnan(out).any()


def test_block_attn_strided_views_and_paper_layout(lib):
    """Tensors handed over in the paper's (N, H, D) token-major layout through the strides."""
    B, H, S, D = 1, 4, 192, 128
    qb, kb, vb = rand_bits((B, S, H, D), 10), rand_bits((B, S, H, D), 11), rand_bits((B, S, H, D), 12)
    q, k, v = (bits_to_dev(x).permute(0, 2, 1, 3) for x in (qb, kb, vb))      # [B,H,S,D] views, stride_s = H*D
    out = torch.zeros((B, S, H, D), dtype=torch.float32, device="cuda").permute(0, 2, 1, 3)
    lse = torch.zeros((B, H, S), dtype=torch.float32, device="cuda")
    lib.tr_block_attn(q, k, v, lib.TR_MASK_NONE, 0.09, out, lse)
    torch.cuda.synchronize()
    tr = lambda x: np.transpose(f64(x), (0, 2, 1, 3))
    ref_o, ref_l = oracle.attention_block(tr(qb), tr(kb), tr(vb), 0.09)
    assert max_abs(to_np(out), ref_o) <= OUT_TOL and max_abs(to_np(lse), ref_l) <= LSE_TOL


def test_block_attn_empty_and_degenerate(lib):
    D = 128
    q = torch.zeros((1, 2, 16, D), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((1, 2, 0, D), dtype=torch.bfloat16, device="cuda")
    out = torch.full((1, 2, 16, D), 7.0, dtype=torch.float32, device="cuda")
    lse = torch.full((1, 2, 16), 7.0, dtype=torch.float32, device="cuda")
    lib.tr_block_attn(q, k, k, lib.TR_MASK_NONE, 1.0, out, lse)            # no keys: identity element
    torch.cuda.synchronize()
    assert torch.all(out == 0) and torch.all(torch.isneginf(lse))
    q0 = torch.zeros((1, 2, 0, D), dtype=torch.bfloat16, device="cuda")     # no queries: nothing to do
    k1 = torch.zeros((1, 2, 8, D), dtype=torch.bfloat16, device="cuda")
    lib.tr_block_attn(q0, k1, k1, lib.TR_MASK_NONE, 1.0, torch.zeros((1, 2, 0, D), device="cuda"),
                      torch.zeros((1, 2, 0), device="cuda"))
    # zero queries: out = mean of values, lse = ln(Sk)
    vb = rand_bits((1, 2, 100, D), 13)
    qz = torch.zeros((1, 2, 40, D), dtype=torch.bfloat16, device="cuda")
    out = torch.empty((1, 2, 40, D), dtype=torch.float32, device="cuda")
    lse = torch.empty((1, 2, 40), dtype=torch.float32, device="cuda")
    lib.tr_block_attn(qz, bits_to_dev(rand_bits((1, 2, 100, D), 14)), bits_to_dev(vb), lib.TR_MASK_NONE, 0.5, out, lse)
    torch.cuda.synchronize()
    # P = 1 exactly for every key, so only the fp32 accumulation order differs
    assert max_abs(to_np(out), np.broadcast_to(f64(vb).mean(axis=2, keepdims=True), (1, 2, 40, D))) <= 1e-5
    assert max_abs(to_np(lse), np.full((1, 2, 40), np.log(100.0))) <= 1e-5


def test_block_attn_large_scores_stay_finite(lib):
    """Scores of several hundred in magnitude: the running-max shift must keep exp() in range."""
    B, H, S, D = 1, 1, 256, 128
    qb, kb, vb = rand_bits((B, H, S, D), 15, std=6.0), rand_bits((B, H, S, D), 16, std=6.0), rand_bits((B, H, S, D), 17)
    out, lse = _run_block(lib, qb, kb, vb, 1.0, lib.TR_MASK_NONE, torch.float32)
    ref_o, ref_l = oracle.attention_block(f64(qb), f64(kb), f64(vb), 1.0)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    assert max_abs(out, ref_o) <= OUT_TOL and max_abs(lse, ref_l) <= LSE_TOL + 1e-6 * np.abs(ref_l).max()


def test_block_attn_is_deterministic(lib):
    qb, kb, vb = rand_bits((1, 4, 512, 128), 18), rand_bits((1, 4, 512, 128), 19), rand_bits((1, 4, 512, 128), 20)
    a = _run_block(lib, qb, kb, vb, 0.088, lib.TR_MASK_CAUSAL_DIAG, torch.float32)
    b = _run_block(lib, qb, kb, vb, 0.088, lib.TR_MASK_CAUSAL_DIAG, torch.float32)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        D = int(rng.choice([64, 128]))
        Hkv = int(rng.choice([1, 2, 3]))
        G = int(rng.choice([1, 2, 4]))
        # key counts around every tile-count boundary of the 4-deep 64-key ring (1 .. 10 tiles) and ragged tails
        Sk = int(rng.choice([int(rng.integers(1, 70)), 64 * int(rng.integers(1, 10)) + int(rng.integers(-2, 3)), int(rng.integers(1, 700))]))
        Sq = int(rng.choice([int(rng.integers(1, 40)), 256 * int(rng.integers(1, 3)) + int(rng.integers(-3, 4)), int(rng.integers(1, 600))]))
        kind = int(rng.integers(0, 3))          # 0 none, 1 causal at random positions, 2 fused Update (no mask)
        q_pos0, k_pos0 = (int(rng.integers(0, 400)), int(rng.integers(0, 400))) if kind == 1 else (0, 0)
        cases.append((i, D, Hkv, G, max(Sq, 1), max(Sk, 1), kind, q_pos0, k_pos0))
    return cases


@pytest.mark.parametrize("case", _random_cases(36, 20260), ids=lambda c: f"{c[0]}-D{c[1]}-Hkv{c[2]}x{c[3]}-Sq{c[4]}-Sk{c[5]}-k{c[6]}")
def test_block_attn_seeded_random_shapes(lib, case):
    """Seeded sweep over shapes that straddle wave, tile and ring-depth boundaries, with GQA, causal offsets
    and the fused Update epilogue; every element is compared with the oracle."""
    i, D, Hkv, G, Sq, Sk, kind, q_pos0, k_pos0 = case
    B, Hq, scale = 1, Hkv * G, 1.0 / np.sqrt(D)
    qb, kb, vb = rand_bits((B, Hq, Sq, D), 500 + 3 * i), rand_bits((B, Hkv, Sk, D), 501 + 3 * i), rand_bits((B, Hkv, Sk, D), 502 + 3 * i)
    if kind == 2:
        rng = np.random.default_rng(900 + i)
        acc_o = rng.standard_normal((B, Hq, Sq, D)).astype(np.float32)
        acc_l = rng.uniform(-5, 15, (B, Hq, Sq)).astype(np.float32)
        acc_l[:, :, ::7] = -np.inf                                   # some empty accumulator rows
        o = torch.from_numpy(acc_o).to("cuda"); l = torch.from_numpy(acc_l).to("cuda")
        lib.tr_block_attn_merge(bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb), lib.TR_MASK_NONE, scale, o, l)
        torch.cuda.synchronize()
        blk_o, blk_l = oracle.attention_block(f64(qb), f64(kb), f64(vb), scale)
        clean = np.where(np.isneginf(acc_l)[..., None], 0.0, acc_o)
        ref_o, ref_l = oracle.merge_pair(clean, acc_l, blk_o, blk_l)
        out, lse = to_np(o), to_np(l)
    elif kind == 1:
        out, lse = _run_block(lib, qb, kb, vb, scale, None, torch.float32, causal_at=(q_pos0, k_pos0))
        ref_o, ref_l = oracle.attention_block(f64(qb), f64(kb), f64(vb), scale, causal_diag=True, q_offset=q_pos0, k_offset=k_pos0)
    else:
        out, lse = _run_block(lib, qb, kb, vb, scale, lib.TR_MASK_NONE, torch.float32)
        ref_o, ref_l = oracle.attention_block(f64(qb), f64(kb), f64(vb), scale)
    assert not np.isnan(out).any() and not np.isnan(lse).any()
    assert max_abs(out, ref_o) <= OUT_TOL and max_abs(lse, ref_l) <= LSE_TOL


@pytest.mark.parametrize("profile", ["rising", "falling", "late_spike", "early_spike", "plateaus"])
def test_block_attn_adversarial_score_profiles(lib, profile):
    """Score profiles along the keys that stress the exponent reference of the softmax: a reference taken early
    must be raised again and again (rising), must not be lost to underflow (falling), and a single late or
    early outlier must take over / keep the row."""
    B, H, Sq, Sk, D = 1, 2, 96, 330, 128
    rng = np.random.default_rng(77)
    q = np.zeros((B, H, Sq, D), dtype=np.float32)
    k = (rng.standard_normal((B, H, Sk, D)) * 0.05).astype(np.float32)
    v = rng.standard_normal((B, H, Sk, D)).astype(np.float32)
    q[..., 0] = 1.0 + (np.arange(Sq) % 5)[None, None, :] * 0.25            # rows differ a little
    q[..., 1:] = (rng.standard_normal((B, H, Sq, D - 1)) * 0.05).astype(np.float32)
    c = np.arange(Sk, dtype=np.float32)
    ramp = {"rising": 0.5 * c, "falling": -0.5 * c,
            "late_spike": np.where(c == Sk - 7, 220.0, 0.0), "early_spike": np.where(c == 3, 220.0, 0.0),
            "plateaus": 40.0 * np.floor(c / 50.0)}[profile].astype(np.float32)
    k[..., 0] = ramp[None, None, :]
    qb, kb, vb = (wl.f32_to_bf16_bits(x) for x in (q, k, v))
    out, lse = _run_block(lib, qb, kb, vb, 1.0, lib.TR_MASK_NONE, torch.float32)
    ref_o, ref_l = oracle.attention_block(f64(qb), f64(kb), f64(vb), 1.0)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    assert max_abs(out, ref_o) <= OUT_TOL
    assert max_abs(lse, ref_l) <= LSE_TOL + 2e-6 * np.abs(ref_l).max()      # fp32 lse of magnitude up to a few hundred
