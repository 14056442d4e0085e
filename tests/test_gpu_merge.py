"""GPU parity of tr_merge against the fp64 oracle (fp32 inputs: max-abs 1e-5)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from gpu_util import max_abs, to_np

pytestmark = pytest.mark.gpu
TOL = 1e-5


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda")


@pytest.mark.parametrize("shape", [(1, 2, 64, 64), (2, 3, 77, 128), (1, 1, 1, 4), (1, 5, 1000, 36)])
def test_merge_pair_matches_oracle(lib, shape):
    B, H, S, D = shape
    rng = np.random.default_rng(1)
    a, b = rng.standard_normal(shape).astype(np.float32), rng.standard_normal(shape).astype(np.float32)
    la, lb = (rng.uniform(-5, 15, (B, H, S)).astype(np.float32) for _ in range(2))
    acc_o, acc_l = _dev(a), _dev(la)
    lib.tr_merge(acc_o, acc_l, _dev(b), _dev(lb))
    torch.cuda.synchronize()
    ref_o, ref_l = oracle.merge_pair(a, la, b, lb)
    assert max_abs(to_np(acc_o), ref_o) <= TOL and max_abs(to_np(acc_l), ref_l) <= TOL
    # and equal to the Update equations as printed in the paper (finite inputs)
    p_o, p_l = oracle.merge_pair_sigmoid_form(a, la, b, lb)
    assert max_abs(to_np(acc_o), p_o) <= TOL and max_abs(to_np(acc_l), p_l) <= TOL


def test_merge_identity_element_and_extremes(lib):
    B, H, S, D = 1, 2, 8, 16
    rng = np.random.default_rng(2)
    a, b = rng.standard_normal((B, H, S, D)).astype(np.float32), rng.standard_normal((B, H, S, D)).astype(np.float32)
    la = rng.uniform(-5, 15, (B, H, S)).astype(np.float32)
    lb = la.copy()
    la[0, 0, 0] = -np.inf                      # empty accumulator row (its out is garbage on purpose)
    a[0, 0, 0] = np.nan
    lb[0, 0, 1] = -np.inf                      # empty block row
    la[0, 0, 2] = lb[0, 0, 2] = -np.inf        # both empty
    lb[0, 0, 3] = la[0, 0, 3] + 200.0          # block dominates
    lb[0, 0, 4] = la[0, 0, 4] - 200.0          # accumulator dominates
    acc_o, acc_l = _dev(a), _dev(la)
    lib.tr_merge(acc_o, acc_l, _dev(b), _dev(lb))
    torch.cuda.synchronize()
    o, l = to_np(acc_o), to_np(acc_l)
    a_clean = a.copy(); a_clean[0, 0, 0] = 0.0
    ref_o, ref_l = oracle.merge_pair(a_clean, la, b, lb)
    assert not np.isnan(o).any() and not np.isnan(l).any()
    assert max_abs(o, ref_o) <= TOL and max_abs(l, ref_l) <= TOL
    assert np.array_equal(o[0, 0, 0], b[0, 0, 0]) and l[0, 0, 0] == lb[0, 0, 0]
    assert np.array_equal(o[0, 0, 1], a[0, 0, 1]) and l[0, 0, 1] == la[0, 0, 1]
    assert np.all(o[0, 0, 2] == 0) and np.isneginf(l[0, 0, 2])
    # self-merge: out unchanged, lse + ln 2
    acc_o, acc_l = _dev(b), _dev(lb)
    lib.tr_merge(acc_o, acc_l, _dev(b), _dev(lb))
    torch.cuda.synchronize()
    fin = np.isfinite(lb)
    assert max_abs(to_np(acc_o)[fin], b[fin]) <= 1e-6 and max_abs(to_np(acc_l)[fin], lb[fin] + np.log(2.0)) <= 1e-5


def test_merge_bf16_block_and_strided_accumulator(lib):
    B, H, S, D = 2, 3, 50, 64
    rng = np.random.default_rng(3)
    a = rng.standard_normal((B, H, S, D)).astype(np.float32)
    bb = wl.f32_to_bf16_bits(rng.standard_normal((B, H, S, D)).astype(np.float32))
    la, lb = (rng.uniform(-5, 15, (B, H, S)).astype(np.float32) for _ in range(2))
    # accumulator is a chunk view of a longer sequence (stride_h > S*D), as inside the ring schedule
    big_o = torch.zeros((B, H, 3 * S, D), dtype=torch.float32, device="cuda")
    big_l = torch.zeros((B, H, 3 * S), dtype=torch.float32, device="cuda")
    acc_o, acc_l = big_o[:, :, S:2 * S], big_l[:, :, S:2 * S]
    acc_o.copy_(_dev(a)); acc_l.copy_(_dev(la))
    blk = torch.from_numpy(bb.view(np.int16)).to("cuda").view(torch.bfloat16)
    lib.tr_merge(acc_o, acc_l, blk, _dev(lb))
    torch.cuda.synchronize()
    ref_o, ref_l = oracle.merge_pair(a, la, wl.bf16_bits_to_f64(bb), lb)
    assert max_abs(to_np(acc_o), ref_o) <= TOL and max_abs(to_np(acc_l), ref_l) <= TOL
    assert torch.all(big_o[:, :, :S] == 0) and torch.all(big_o[:, :, 2 * S:] == 0)       # neighbours untouched
    assert torch.all(big_l[:, :, :S] == 0) and torch.all(big_l[:, :, 2 * S:] == 0)


def test_merge_empty(lib):
    z4 = torch.zeros((1, 2, 0, 64), device="cuda"); z3 = torch.zeros((1, 2, 0), device="cuda")
    lib.tr_merge(z4, z3, z4.clone(), z3.clone())


def test_merge_config4_downscaled_ring_order_and_any_order(lib):
    """Eight partials merged in ring order 0..7 from the identity; any other order agrees too."""
    cfg = wl.CONFIGS["cfg4_merge"]
    S = 512
    outs, lses = wl.make_merge_partials(cfg, S=S)
    ref_o, ref_l = oracle.merge_nary(outs, lses)
    for order in (list(range(8)), [7, 3, 0, 5, 1, 6, 2, 4]):
        acc_o = torch.zeros((cfg.B, cfg.H, S, cfg.D), dtype=torch.float32, device="cuda")
        acc_l = torch.full((cfg.B, cfg.H, S), float("-inf"), dtype=torch.float32, device="cuda")
        for i in order:
            lib.tr_merge(acc_o, acc_l, _dev(outs[i]), _dev(lses[i]))
        torch.cuda.synchronize()
        assert max_abs(to_np(acc_o), ref_o) <= TOL and max_abs(to_np(acc_l), ref_l) <= TOL


# ---------------------------------------------------------------- n-ary merge (the Update folded over n partials)
def _bf16_round(x):
    return wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(x))


@pytest.mark.parametrize("n", [1, 2, 3, 8, 16])
@pytest.mark.parametrize("shape,bf16", [((1, 2, 77, 128), False), ((2, 3, 130, 64), True), ((1, 5, 1000, 36), False), ((1, 2, 33, 40), True)])
@pytest.mark.parametrize("accumulate", [False, True])
def test_merge_n_matches_oracle(lib, n, shape, bf16, accumulate):
    B, H, S, D = shape
    rng = np.random.default_rng(100 + n)
    outs = [rng.standard_normal(shape).astype(np.float32) for _ in range(n)]
    if bf16:
        outs = [_bf16_round(o) for o in outs]
    lses = [rng.uniform(-5, 15, (B, H, S)).astype(np.float32) for _ in range(n)]
    for i in range(n):                                      # sprinkle empty rows; row 0 is empty everywhere
        lses[i][rng.random((B, H, S)) < 0.1] = -np.inf
        lses[i][:, :, 0] = -np.inf
        outs[i][np.isneginf(lses[i])] = np.nan if not bf16 else 0.0   # garbage that must not leak
    old_o = rng.standard_normal(shape).astype(np.float32)
    old_l = rng.uniform(-5, 15, (B, H, S)).astype(np.float32)
    old_l[:, :, 0] = -np.inf
    out, lse = (_dev(old_o), _dev(old_l)) if accumulate else (torch.full(shape, float("nan"), device="cuda"), torch.full((B, H, S), float("nan"), device="cuda"))
    dev_o = [(_dev(o).to(torch.bfloat16) if bf16 else _dev(o)) for o in outs]
    lib.tr_merge_n(out, lse, dev_o, [_dev(l) for l in lses], accumulate)
    torch.cuda.synchronize()
    clean = [np.where(np.isneginf(l)[..., None], 0.0, o) for o, l in zip(outs, lses)]
    ref_o, ref_l = oracle.merge_nary(clean + ([old_o] if accumulate else []), lses + ([old_l] if accumulate else []))
    o, l = to_np(out), to_np(lse)
    assert not np.isnan(o).any() and not np.isnan(l).any()
    assert max_abs(o, ref_o) <= TOL and max_abs(l, ref_l) <= TOL
    assert np.all(o[:, :, 0] == 0) and np.all(np.isneginf(l[:, :, 0]))       # all partials empty: identity element


def test_merge_n_agrees_with_pairwise_updates(lib):
    """Folding tr_merge over the partials (Algorithm 1's way) and the one-pass form agree to rounding."""
    B, H, S, D, n = 1, 4, 300, 128, 8
    rng = np.random.default_rng(7)
    outs = [_dev(rng.standard_normal((B, H, S, D)).astype(np.float32)) for _ in range(n)]
    lses = [_dev(rng.uniform(-5, 15, (B, H, S)).astype(np.float32)) for _ in range(n)]
    acc_o = torch.zeros((B, H, S, D), device="cuda"); acc_l = torch.full((B, H, S), float("-inf"), device="cuda")
    for o, l in zip(outs, lses):
        lib.tr_merge(acc_o, acc_l, o, l)
    one_o = torch.empty_like(acc_o); one_l = torch.empty_like(acc_l)
    lib.tr_merge_n(one_o, one_l, outs, lses)
    torch.cuda.synchronize()
    assert max_abs(to_np(one_o), to_np(acc_o)) <= TOL and max_abs(to_np(one_l), to_np(acc_l)) <= TOL


def test_merge_n_argument_errors(lib):
    o = torch.zeros((1, 2, 8, 16), device="cuda"); l = torch.zeros((1, 2, 8), device="cuda")
    b = [torch.zeros((1, 2, 8, 16), device="cuda") for _ in range(17)]; bl = [torch.zeros((1, 2, 8), device="cuda") for _ in range(17)]
    with pytest.raises(lib.TokenRingError, match="out of range"):
        lib.tr_merge_n(o, l, b, bl)
    with pytest.raises(lib.TokenRingError, match="out of range"):
        lib.tr_merge_n(o, l, [], [])
    with pytest.raises(lib.TokenRingError, match="overlaps"):
        lib.tr_merge_n(o, l, [b[0], o], [bl[0], bl[1]])
    with pytest.raises(lib.TokenRingError, match="one dtype"):
        lib.tr_merge_n(o, l, [b[0], b[1].to(torch.bfloat16)], bl[:2])
    with pytest.raises(lib.TokenRingError, match="share their strides"):
        lib.tr_merge_n(o, l, [b[0], torch.zeros((1, 2, 8, 32), device="cuda")[..., :16]], bl[:2])
    with pytest.raises(lib.TokenRingError, match="shape"):
        lib.tr_merge_n(o, l, [b[0], torch.zeros((1, 2, 9, 16), device="cuda")], bl[:2])
