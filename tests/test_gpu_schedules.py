"""GPU parity of tr_ring_attn_sched: every step order (Algorithm 1, Ring Attention of Sec. 2.1,
the zigzag partition of Sec. 3.3.2, the two-level scheme of Sec. 3.3.3) must reach unchunked
fp64 attention within max-abs 1e-2 on out and 1e-3 on lse; the orders differ only in fp32
rounding of the merge sequence."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from gpu_util import bits_to_dev, check_rows as _check_rows, f64, max_abs, rand_bits, to_np

pytestmark = pytest.mark.gpu
OUT_TOL, LSE_TOL = 1e-2, 1e-3


def _sched(lib, q, k, v, n_dev, causal, schedule, n_inner=1, scale=0.0):
    B, Hq, S, D = q.shape
    out = torch.full((B, Hq, S, D), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((B, Hq, S), float("nan"), dtype=torch.float32, device="cuda")
    lib.tr_ring_attn_sched(q, k, v, n_dev, causal, schedule, out, lse, scale, n_inner)
    torch.cuda.synchronize()
    return out, lse


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("name,n_dev,n_inner", [("tokenring", 4, 1), ("ring", 4, 1), ("zigzag", 4, 1), ("zigzag", 1, 1),
                                                ("hybrid", 8, 4), ("hybrid", 6, 2), ("hybrid", 4, 4), ("hybrid", 4, 1)])
def test_every_schedule_reaches_unchunked_attention(lib, name, n_dev, n_inner, causal):
    if name == "zigzag" and not causal:
        pytest.skip("the zigzag partition is causal by definition")
    schedule = {"tokenring": lib.TR_SCHED_TOKENRING, "ring": lib.TR_SCHED_RING_ATTENTION,
                "zigzag": lib.TR_SCHED_ZIGZAG, "hybrid": lib.TR_SCHED_HYBRID}[name]
    B, Hq, Hkv, S, D = 2, 4, 2, 480, 128          # 480 = 8*60 = 6*80 = 4*120: ragged tiles in every segment
    qb, kb, vb = rand_bits((B, Hq, S, D), 41), rand_bits((B, Hkv, S, D), 42), rand_bits((B, Hkv, S, D), 43)
    out, lse = _sched(lib, bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb), n_dev, causal, schedule, n_inner)
    ref_o, ref_l = oracle.attention_full(f64(qb), f64(kb), f64(vb), 1.0 / np.sqrt(D), causal)
    assert max_abs(to_np(out), ref_o) <= OUT_TOL and max_abs(to_np(lse), ref_l) <= LSE_TOL


@pytest.mark.parametrize("D,n_dev,seg", [(128, 2, 128), (128, 3, 384), (128, 4, 256), (64, 2, 128), (64, 3, 384), (64, 5, 256)])
def test_zigzag_attends_the_k_v_pair_of_a_device_in_one_step(lib, D, n_dev, seg):
    """Segments that are whole K/V tiles: the later Query segment of a pair meets both K/V segments of a
    device in one block step whose key range changes segment between two tiles (Sec. 3.3.2 partition,
    attention and its log-sum-exp, Sec. 3.1, over the concatenated keys); on iteration 0 the second half carries the diagonal mask."""
    B, Hq, Hkv, S = 2, 4, 2, 2 * n_dev * seg
    qb, kb, vb = rand_bits((B, Hq, S, D), 61), rand_bits((B, Hkv, S, D), 62), rand_bits((B, Hkv, S, D), 63)
    out, lse = _sched(lib, bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb), n_dev, True, lib.TR_SCHED_ZIGZAG, 1)
    ref_o, ref_l = oracle.attention_full(f64(qb), f64(kb), f64(vb), 1.0 / np.sqrt(D), True)
    assert max_abs(to_np(out), ref_o) <= OUT_TOL and max_abs(to_np(lse), ref_l) <= LSE_TOL
    steps = lib.tr_schedule_steps(lib.TR_SCHED_ZIGZAG, n_dev, True)
    assert max(g for _, _, g in steps) + 1 == n_dev          # one launch per iteration


def _random_schedule_cases(n_cases, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n_cases):
        sched = int(rng.integers(0, 4))
        n_dev = int(rng.choice([1, 2, 3, 4, 6, 8]))
        n_inner = 1
        if sched == 3:
            n_inner = int(rng.choice([d for d in (1, 2, 3, 4) if n_dev % d == 0]))
        causal = True if sched == 2 else bool(rng.integers(0, 2))
        seg = int(rng.choice([40, 64, 128, 128, 256, 384]))          # 128-multiples take the paired zigzag steps
        n_seg = 2 * n_dev if sched == 2 else n_dev
        while n_seg * seg > 3072:
            seg //= 2
        D = int(rng.choice([64, 128]))
        Hkv = int(rng.choice([1, 2, 8]))
        G = int(rng.choice([1, 2, 3]))
        B = int(rng.choice([1, 2])) if Hkv < 8 else 1
        cases.append((i, sched, n_dev, n_inner, causal, seg, D, Hkv, G, B))
    return cases


@pytest.mark.parametrize("case", _random_schedule_cases(28, 20261),
                         ids=lambda c: f"{c[0]}-sched{c[1]}-n{c[2]}x{c[3]}-{'causal' if c[4] else 'full'}-seg{c[5]}-D{c[6]}-Hkv{c[7]}x{c[8]}-B{c[9]}")
def test_seeded_random_schedules_reach_unchunked_attention(lib, case):
    """Seeded sweep over schedule, device count, segment length (ragged and whole tiles), head dim, GQA group
    (including 3) and batch: every combination must reach unchunked fp64 attention."""
    i, sched, n_dev, n_inner, causal, seg, D, Hkv, G, B = case
    n_seg = 2 * n_dev if sched == 2 else n_dev
    S, Hq = n_seg * seg, Hkv * G
    qb, kb, vb = rand_bits((B, Hq, S, D), 700 + 3 * i), rand_bits((B, Hkv, S, D), 701 + 3 * i), rand_bits((B, Hkv, S, D), 702 + 3 * i)
    out, lse = _sched(lib, bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb), n_dev, causal, sched, n_inner)
    ref_o, ref_l = oracle.attention_full(f64(qb), f64(kb), f64(vb), 1.0 / np.sqrt(D), causal)
    assert max_abs(to_np(out), ref_o) <= OUT_TOL and max_abs(to_np(lse), ref_l) <= LSE_TOL


def test_tokenring_schedule_is_tr_ring_attn_bitwise(lib):
    qb, kb, vb = rand_bits((1, 4, 1024, 64), 44), rand_bits((1, 4, 1024, 64), 45), rand_bits((1, 4, 1024, 64), 46)
    q, k, v = bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb)
    for causal in (False, True):
        a = _sched(lib, q, k, v, 4, causal, lib.TR_SCHED_TOKENRING)
        out = torch.empty_like(a[0]); lse = torch.empty_like(a[1])
        lib.tr_ring_attn(q, k, v, 4, causal, out, lse, 0.0, None)
        torch.cuda.synchronize()
        assert torch.equal(a[0], out) and torch.equal(a[1], lse)
        # one-node hybrid is Algorithm 1 as well, all-singleton nodes are Ring Attention
        h = _sched(lib, q, k, v, 4, causal, lib.TR_SCHED_HYBRID, n_inner=4)
        r = _sched(lib, q, k, v, 4, causal, lib.TR_SCHED_RING_ATTENTION)
        h1 = _sched(lib, q, k, v, 4, causal, lib.TR_SCHED_HYBRID, n_inner=1)
        assert torch.equal(a[0], h[0]) and torch.equal(a[1], h[1])
        assert torch.equal(r[0], h1[0]) and torch.equal(r[1], h1[1])


def test_schedule_argument_errors(lib):
    q = bits_to_dev(rand_bits((1, 2, 256, 64), 47))
    out = torch.empty((1, 2, 256, 64), dtype=torch.float32, device="cuda"); lse = torch.empty((1, 2, 256), device="cuda")
    with pytest.raises(lib.TokenRingError, match="zigzag"):
        lib.tr_ring_attn_sched(q, q, q, 4, False, lib.TR_SCHED_ZIGZAG, out, lse)
    with pytest.raises(lib.TokenRingError, match="n_inner"):
        lib.tr_ring_attn_sched(q, q, q, 4, True, lib.TR_SCHED_HYBRID, out, lse, 0.0, 3)
    with pytest.raises(lib.TokenRingError, match="segments"):
        lib.tr_ring_attn_sched(q, q, q, 3, True, lib.TR_SCHED_ZIGZAG, out, lse)      # 256 % 6 != 0
    with pytest.raises(lib.TokenRingError, match="unknown schedule"):
        lib.tr_ring_attn_sched(q, q, q, 4, True, 9, out, lse)


@pytest.mark.parametrize("name,n_inner", [("zigzag", 1), ("hybrid", 4), ("ring", 1)])
def test_config3_shape_other_schedules_sampled_rows(lib, name, n_inner):
    """cfg3 (causal, S = 32768, 8 devices): zigzag over 16 segments of 2048, 2 nodes x 4 devices, Ring Attention order."""
    cfg = wl.CONFIGS["cfg3_ring"]
    qb, kb, vb = wl.make_qkv_bits(cfg)
    schedule = {"zigzag": lib.TR_SCHED_ZIGZAG, "hybrid": lib.TR_SCHED_HYBRID, "ring": lib.TR_SCHED_RING_ATTENTION}[name]
    out, lse = _sched(lib, bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb), cfg.n_chunks, True, schedule, n_inner, cfg.scale)
    assert not torch.isnan(out).any() and not torch.isnan(lse).any()
    worst_o, worst_l, n = _check_rows(cfg, out, lse, qb, kb, vb, n_random=128)
    print(f"cfg3 {name}: {n} rows x {cfg.Hq} heads, max|d out| {worst_o:.3e}, max|d lse| {worst_l:.3e}")
    assert worst_o <= OUT_TOL and worst_l <= LSE_TOL
