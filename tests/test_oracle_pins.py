"""Pins of the fp64 oracle against things other than itself (CPU only).

Each test is chosen so that a plausible mistake in the oracle - a dropped scale, a wrong
mask direction, a transposed operand, a missing max-shift term, a wrong GQA mapping, a
sign error in the Update - fails at least one of them.
"""
import os

import mpmath as mp
import numpy as np
import pytest
import scipy.special
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed, std=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * std


# ---------------------------------------------------------------- brute force, 50 digits
def _mp_attention(q, k, v, scale, causal):
    """Row-by-row softmax attention in 50-digit arithmetic with python loops (one head)."""
    mp.mp.dps = 50
    Sq, D = q.shape
    Sk = k.shape[0]
    out = np.zeros((Sq, D))
    lse = np.zeros(Sq)
    for r in range(Sq):
        keys = [c for c in range(Sk) if (not causal or c <= r)]
        s = [mp.mpf(scale) * sum(mp.mpf(float(q[r, d])) * mp.mpf(float(k[c, d])) for d in range(D)) for c in keys]
        z = sum(mp.e ** x for x in s)
        lse[r] = float(mp.log(z))
        for d in range(D):
            out[r, d] = float(sum((mp.e ** x) / z * mp.mpf(float(v[c, d])) for x, c in zip(s, keys)))
    return out, lse


@pytest.mark.parametrize("causal", [False, True])
def test_attention_matches_mpmath_bruteforce(causal):
    B, Hq, Hkv, S, D = 1, 2, 1, 8, 4
    q, k, v = _rand((B, Hq, S, D), 1), _rand((B, Hkv, S, D), 2), _rand((B, Hkv, S, D), 3)
    scale = 0.37
    out, lse = oracle.attention_full(q, k, v, scale, causal)
    for h in range(Hq):
        o_ref, l_ref = _mp_attention(q[0, h], k[0, 0], v[0, 0], scale, causal)
        assert np.max(np.abs(out[0, h] - o_ref)) < 1e-13
        assert np.max(np.abs(lse[0, h] - l_ref)) < 1e-13


def test_non_square_block_matches_mpmath():
    q, k, v = _rand((1, 1, 5, 3), 4), _rand((1, 1, 9, 3), 5), _rand((1, 1, 9, 3), 6)
    out, lse = oracle.attention_block(q, k, v, 1.3)
    o_ref, l_ref = _mp_attention(q[0, 0], k[0, 0], v[0, 0], 1.3, False)
    assert np.max(np.abs(out[0, 0] - o_ref)) < 1e-13 and np.max(np.abs(lse[0, 0] - l_ref)) < 1e-13


def _mp_attention_at(q, k, v, scale, q_pos, k_pos):
    """50-digit brute force with explicit sequence positions: key c is visible to row r iff
    k_pos[c] <= q_pos[r] (Sec. 3.3.2).  A row that sees no key is the empty sum: out = 0, lse = -inf."""
    mp.mp.dps = 50
    out = np.zeros((len(q_pos), v.shape[1]))
    lse = np.full(len(q_pos), -np.inf)
    for r, qp in enumerate(q_pos):
        keys = [c for c, kp in enumerate(k_pos) if kp <= qp]
        if not keys:
            continue
        s = [mp.mpf(scale) * sum(mp.mpf(float(q[r, d])) * mp.mpf(float(k[c, d])) for d in range(q.shape[1])) for c in keys]
        z = sum(mp.e ** x for x in s)
        lse[r] = float(mp.log(z))
        for d in range(v.shape[1]):
            out[r, d] = float(sum((mp.e ** x) / z * mp.mpf(float(v[c, d])) for x, c in zip(s, keys)))
    return out, lse


@pytest.mark.parametrize("q_offset,k_offset,Sq,Sk", [(0, 3, 8, 8), (2, 5, 8, 6), (5, 2, 7, 8), (0, 8, 4, 4), (4, 0, 3, 9)])
def test_causal_block_at_offsets_matches_mpmath(q_offset, k_offset, Sq, Sk):
    """The causal rule at arbitrary chunk positions, as the zigzag partition of Sec. 3.3.2 needs it:
    K/V chunks that start after the Query chunk leave early rows with few keys or none."""
    D = 3
    q, k, v = _rand((1, 1, Sq, D), 40 + q_offset), _rand((1, 1, Sk, D), 50 + k_offset), _rand((1, 1, Sk, D), 60)
    out, lse = oracle.attention_block(q, k, v, 0.8, causal_diag=True, q_offset=q_offset, k_offset=k_offset)
    o_ref, l_ref = _mp_attention_at(q[0, 0], k[0, 0], v[0, 0], 0.8, q_offset + np.arange(Sq), k_offset + np.arange(Sk))
    empty = np.isneginf(l_ref)
    # rows without a visible key: exactly the identity element of the Update
    n_empty = sum(1 for r in range(Sq) if q_offset + r < k_offset)
    assert empty.sum() == n_empty
    assert np.all(np.isneginf(lse[0, 0][empty])) and np.all(out[0, 0][empty] == 0.0)
    assert np.max(np.abs(out[0, 0] - o_ref)) < 1e-13
    assert np.max(np.abs(lse[0, 0][~empty] - l_ref[~empty]), initial=0.0) < 1e-13
    # number of visible keys per row, counted by hand: clamp(q_offset + r - k_offset + 1, 0, Sk)
    zq = np.zeros_like(q)
    _, lse0 = oracle.attention_block(zq, k, v, 0.8, causal_diag=True, q_offset=q_offset, k_offset=k_offset)
    count = np.clip(q_offset + np.arange(Sq) - k_offset + 1, 0, Sk)
    with np.errstate(divide="ignore"):
        assert np.allclose(lse0[0, 0], np.log(count), atol=1e-14)


# ---------------------------------------------------------------- library special cases
@pytest.mark.parametrize("causal", [False, True])
def test_attention_matches_torch_sdpa_fp64(causal):
    B, H, S, D = 2, 3, 96, 16
    q, k, v = _rand((B, H, S, D), 7), _rand((B, H, S, D), 8), _rand((B, H, S, D), 9)
    scale = 1.0 / np.sqrt(D)
    out, lse = oracle.attention_full(q, k, v, scale, causal)
    tq, tk, tv = (torch.from_numpy(x) for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=causal, scale=scale).numpy()
    assert np.max(np.abs(out - ref)) < 1e-12
    s = scale * np.einsum("bhqd,bhkd->bhqk", q, k)
    if causal:
        s = np.where(np.tril(np.ones((S, S), dtype=bool)), s, -np.inf)
    assert np.max(np.abs(lse - scipy.special.logsumexp(s, axis=-1))) < 1e-12
    assert np.max(np.abs(lse - torch.logsumexp(torch.from_numpy(s), dim=-1).numpy())) < 1e-12


# ---------------------------------------------------------------- closed forms
def test_zero_queries_give_mean_of_values():
    B, H, S, D = 1, 2, 17, 5
    q = np.zeros((B, H, S, D))
    k, v = _rand((B, H, S, D), 10), _rand((B, H, S, D), 11)
    out, lse = oracle.attention_full(q, k, v, 0.5, False)
    assert np.allclose(out, np.broadcast_to(v.mean(axis=2, keepdims=True), out.shape), atol=1e-14)
    assert np.allclose(lse, np.log(S), atol=1e-14)
    out, lse = oracle.attention_full(q, k, v, 0.5, True)
    prefix_mean = np.cumsum(v, axis=2) / np.arange(1, S + 1)[None, None, :, None]
    assert np.allclose(out, prefix_mean, atol=1e-14)
    assert np.allclose(lse, np.log(np.arange(1, S + 1)), atol=1e-14)


def test_causal_row0_is_v0_and_score00():
    q, k, v = _rand((1, 1, 6, 4), 12), _rand((1, 1, 6, 4), 13), _rand((1, 1, 6, 4), 14)
    out, lse = oracle.attention_full(q, k, v, 0.7, True)
    assert np.allclose(out[0, 0, 0], v[0, 0, 0], atol=1e-15)
    assert np.isclose(lse[0, 0, 0], 0.7 * q[0, 0, 0] @ k[0, 0, 0], atol=1e-15)


def test_equal_keys_shift_lse_by_common_score():
    S, D = 9, 4
    q, v = _rand((1, 1, S, D), 15), _rand((1, 1, S, D), 16)
    k = np.broadcast_to(_rand((1, 1, 1, D), 17), (1, 1, S, D)).copy()
    out, lse = oracle.attention_full(q, k, v, 0.9, False)
    assert np.allclose(out, np.broadcast_to(v.mean(axis=2, keepdims=True), out.shape), atol=1e-13)
    assert np.allclose(lse[0, 0], 0.9 * q[0, 0] @ k[0, 0, 0] + np.log(S), atol=1e-13)


def test_dominant_key_selects_its_value_and_scale_matters():
    S, D = 8, 4
    q = np.zeros((1, 1, 1, D)); q[..., 0] = 1.0
    k = np.zeros((1, 1, S, D)); k[0, 0, 3, 0] = 200.0
    v = _rand((1, 1, S, D), 18)
    out, lse = oracle.attention_block(q, k, v, 1.0)
    assert np.allclose(out[0, 0, 0], v[0, 0, 3], atol=1e-12)
    assert np.isclose(lse[0, 0, 0], 200.0, atol=1e-12)
    # hand value: two keys with scores scale*ln(3) and 0 -> weights 3^scale/(3^scale+1)
    k2 = np.zeros((1, 1, 2, 1)); k2[0, 0, 0, 0] = np.log(3.0)
    v2 = np.array([1.0, 0.0]).reshape(1, 1, 2, 1)
    out, lse = oracle.attention_block(np.ones((1, 1, 1, 1)), k2, v2, 2.0)
    assert np.isclose(out[0, 0, 0, 0], 0.9, atol=1e-15) and np.isclose(lse[0, 0, 0], np.log(10.0), atol=1e-15)


def test_mask_direction_future_keys_do_not_matter():
    q, k, v = _rand((1, 1, 10, 4), 19), _rand((1, 1, 10, 4), 20), _rand((1, 1, 10, 4), 21)
    out, lse = oracle.attention_full(q, k, v, 0.4, True)
    k2, v2 = k.copy(), v.copy()
    k2[0, 0, 6:] += 5.0; v2[0, 0, 6:] -= 3.0          # change only keys at positions >= 6
    out2, lse2 = oracle.attention_full(q, k2, v2, 0.4, True)
    assert np.array_equal(out[0, 0, :6], out2[0, 0, :6]) and np.array_equal(lse[0, 0, :6], lse2[0, 0, :6])
    assert not np.allclose(out[0, 0, 6:], out2[0, 0, 6:])


# ---------------------------------------------------------------- invariants
def test_softmax_rows_sum_to_one_and_reproduce_out():
    q, k, v = _rand((40, 8), 22), _rand((40, 8), 23), _rand((40, 8), 24)
    for causal in (False, True):
        w = oracle.softmax_weights(q, k, 0.35, causal)
        assert np.allclose(w.sum(axis=1), 1.0, atol=1e-14)
        if causal:
            assert np.all(np.triu(w, 1) == 0.0)
        out, _ = oracle.attention_full(q[None, None], k[None, None], v[None, None], 0.35, causal)
        assert np.allclose(w @ v, out[0, 0], atol=1e-14)


def _ring_attention_order(n, causal):
    """Ring Attention's order: Query chunk c stays put and sees K/V chunks c, c-1, c-2, ..."""
    return [(c, (c - i) % n) for i in range(n) for c in range(n) if not (causal and (c - i) % n > c)]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("n_chunks", [1, 2, 4, 8, 32])
def test_chunked_equals_unchunked(n_chunks, causal):
    B, Hq, Hkv, S, D = 1, 4, 2, 32, 8
    q, k, v = _rand((B, Hq, S, D), 25), _rand((B, Hkv, S, D), 26), _rand((B, Hkv, S, D), 27)
    ref_o, ref_l = oracle.attention_full(q, k, v, 0.3, causal)
    o, l = oracle.ring_attention(q, k, v, n_chunks, causal, 0.3)
    assert np.max(np.abs(o - ref_o)) < 1e-13 and np.max(np.abs(l - ref_l)) < 1e-13


@pytest.mark.parametrize("causal", [False, True])
def test_merge_order_invariance(causal):
    B, H, S, D, n = 1, 2, 48, 8, 6
    q, k, v = _rand((B, H, S, D), 28), _rand((B, H, S, D), 29), _rand((B, H, S, D), 30)
    ref_o, ref_l = oracle.attention_full(q, k, v, 0.25, causal)
    token_ring = [(c, j) for (_, j, c) in oracle.ring_schedule(n, causal)]
    ring_attn = _ring_attention_order(n, causal)
    assert sorted(token_ring) == sorted(ring_attn)
    shuffled = list(token_ring)
    np.random.default_rng(31).shuffle(shuffled)
    for order in (token_ring, ring_attn, shuffled, token_ring[::-1]):
        o, l = oracle.ring_attention(q, k, v, n, causal, 0.25, order=order)
        assert np.max(np.abs(o - ref_o)) < 1e-13 and np.max(np.abs(l - ref_l)) < 1e-13
    # tree / n-ary merge of the per-chunk partials of one query chunk
    C = S // n
    c = n - 1
    parts = [oracle.attention_block(q[:, :, c * C:], k[:, :, j * C:(j + 1) * C], v[:, :, j * C:(j + 1) * C], 0.25,
                                    causal_diag=causal, q_offset=c * C, k_offset=j * C) for j in range(n)]
    o, l = oracle.merge_nary([p[0] for p in parts], [p[1] for p in parts])
    assert np.max(np.abs(o - ref_o[:, :, c * C:])) < 1e-13 and np.max(np.abs(l - ref_l[:, :, c * C:])) < 1e-13
    # binary tree of pairwise Updates over the same partials
    level = parts
    while len(level) > 1:
        nxt = [oracle.merge_pair(level[i][0], level[i][1], level[i + 1][0], level[i + 1][1]) for i in range(0, len(level) - 1, 2)]
        level = nxt + ([level[-1]] if len(level) % 2 else [])
    assert np.max(np.abs(level[0][0] - ref_o[:, :, c * C:])) < 1e-13 and np.max(np.abs(level[0][1] - ref_l[:, :, c * C:])) < 1e-13


def test_gqa_equals_mha_with_repeated_kv():
    B, Hq, Hkv, S, D = 1, 8, 2, 24, 8
    q, k, v = _rand((B, Hq, S, D), 32), _rand((B, Hkv, S, D), 33), _rand((B, Hkv, S, D), 34)
    o, l = oracle.attention_full(q, k, v, 0.3, True)
    kr, vr = np.repeat(k, Hq // Hkv, axis=1), np.repeat(v, Hq // Hkv, axis=1)   # heads 0..3 -> kv 0, 4..7 -> kv 1
    o2, l2 = oracle.attention_full(q, kr, vr, 0.3, True)
    assert np.array_equal(o, o2) and np.array_equal(l, l2)
    assert not np.allclose(o[:, 3], oracle.attention_full(q[:, 3:4], k[:, 1:2], v[:, 1:2], 0.3, True)[0][:, 0])


def test_attention_rows_matches_full():
    B, Hq, Hkv, S, D = 1, 4, 2, 200, 8
    q, k, v = _rand((B, Hq, S, D), 35), _rand((B, Hkv, S, D), 36), _rand((B, Hkv, S, D), 37)
    rows = np.array([0, 1, 63, 64, 65, 130, 199])
    for causal in (False, True):
        ref_o, ref_l = oracle.attention_full(q, k, v, 0.3, causal)
        for h in range(Hq):
            o, l = oracle.attention_rows(q[0, h, rows], rows, k[0, h // 2], v[0, h // 2], 0.3, causal)
            assert np.max(np.abs(o - ref_o[0, h, rows])) < 1e-13 and np.max(np.abs(l - ref_l[0, h, rows])) < 1e-13


# ---------------------------------------------------------------- the Update (merge)
def _mp_merge_printed(out, lse, bout, blse):
    """Sec. 3.1's two Update equations evaluated in 50-digit arithmetic."""
    mp.mp.dps = 50
    sig = lambda x: 1 / (1 + mp.e ** (-x))
    o, l, bo, bl = mp.mpf(float(out)), mp.mpf(float(lse)), mp.mpf(float(bout)), mp.mpf(float(blse))
    return float(o - sig(bl - l) * (o - bo)), float(l - mp.log(sig(l - bl)))


def test_merge_matches_printed_update_equations():
    rng = np.random.default_rng(38)
    out, bout = rng.standard_normal((50, 3)), rng.standard_normal((50, 3))
    lse, blse = rng.uniform(-5, 15, 50), rng.uniform(-5, 15, 50)
    o1, l1 = oracle.merge_pair_sigmoid_form(out, lse, bout, blse)
    o2, l2 = oracle.merge_pair(out, lse, bout, blse)
    assert np.max(np.abs(o1 - o2)) < 1e-13 and np.max(np.abs(l1 - l2)) < 1e-13
    for i in range(50):
        o_ref, l_ref = _mp_merge_printed(out[i, 0], lse[i], bout[i, 0], blse[i])
        assert abs(o2[i, 0] - o_ref) < 1e-13 and abs(l2[i] - l_ref) < 1e-13
        assert abs(o1[i, 0] - o_ref) < 1e-13 and abs(l1[i] - l_ref) < 1e-13


def test_merge_algebra():
    rng = np.random.default_rng(39)
    a, b, c = (rng.standard_normal((20, 4)) for _ in range(3))
    la, lb, lc = (rng.uniform(-5, 15, 20) for _ in range(3))
    zero, ninf = np.zeros((20, 4)), np.full(20, -np.inf)
    # identity element on either side, and identity with identity
    for o, l in (oracle.merge_pair(zero, ninf, a, la), oracle.merge_pair(a, la, zero, ninf)):
        assert np.array_equal(o, a) and np.array_equal(l, la)
    o, l = oracle.merge_pair(zero, ninf, zero, ninf)
    assert np.array_equal(o, zero) and np.all(np.isneginf(l))
    # a block merged with itself: out unchanged, lse + ln 2
    o, l = oracle.merge_pair(a, la, a, la)
    assert np.allclose(o, a, atol=1e-15) and np.allclose(l, la + np.log(2.0), atol=1e-14)
    # commutative, associative, and equal to the n-ary definition
    o_ab, l_ab = oracle.merge_pair(a, la, b, lb)
    o_ba, l_ba = oracle.merge_pair(b, lb, a, la)
    assert np.allclose(o_ab, o_ba, atol=1e-14) and np.allclose(l_ab, l_ba, atol=1e-14)
    o1, l1 = oracle.merge_pair(*oracle.merge_pair(a, la, b, lb), c, lc)
    o2, l2 = oracle.merge_pair(a, la, *oracle.merge_pair(b, lb, c, lc))
    o3, l3 = oracle.merge_nary([a, b, c], [la, lb, lc])
    assert np.allclose(o1, o2, atol=1e-14) and np.allclose(l1, l2, atol=1e-14)
    assert np.allclose(o1, o3, atol=1e-14) and np.allclose(l1, l3, atol=1e-14)
    # n-ary definition written with scipy: weights softmax(lse_i), lse = logsumexp
    w = scipy.special.softmax(np.stack([la, lb, lc]), axis=0)
    assert np.allclose(o3, w[0][:, None] * a + w[1][:, None] * b + w[2][:, None] * c, atol=1e-14)
    assert np.allclose(l3, scipy.special.logsumexp(np.stack([la, lb, lc]), axis=0), atol=1e-14)
    # a far larger block lse wins outright; a far smaller one changes nothing
    o, l = oracle.merge_pair(a, la, b, la + 800.0)
    assert np.allclose(o, b, atol=1e-15) and np.array_equal(l, la + 800.0)
    o, l = oracle.merge_pair(a, la, b, la - 800.0)
    assert np.array_equal(o, a) and np.array_equal(l, la)


# ---------------------------------------------------------------- the schedule (paper walk-through)
def test_schedule_matches_four_device_walkthrough():
    rows = [tuple(int(x) for x in line.split()) for line in open(os.path.join(GOLDEN, "walkthrough_4gpu.txt"))
            if line.strip() and not line.startswith("#")]
    steps = oracle.ring_schedule(4, causal=False)
    assert len(steps) == 16 == len(rows)
    for (i, j, c), (step, dev, q_owner, dest_off) in zip(steps, rows):
        assert (i, j, c) == (step, dev, q_owner)
        assert (dev + dest_off) % 4 == c            # the block result travels to the Query chunk's owner


def test_schedule_counts_and_per_chunk_order():
    for n in (1, 4, 8, 16):
        full, causal = oracle.ring_schedule(n, False), oracle.ring_schedule(n, True)
        assert len(full) == n * n and len(causal) == n * (n + 1) // 2
        assert sorted((c, j) for _, j, c in full) == [(c, j) for c in range(n) for j in range(n)]
        assert sorted((c, j) for _, j, c in causal) == [(c, j) for c in range(n) for j in range(c + 1)]
        for c in range(n):   # Query chunk c meets K/V chunks c, c+1, ... (mod n) in that order
            assert [j for _, j, cc in full if cc == c] == [(c + i) % n for i in range(n)]
    assert len(oracle.ring_schedule(8, True)) == 36 and len(oracle.ring_schedule(16, True)) == 136


def test_zigzag_example_from_paper():
    # four devices, eight segments: device 0 processes segments 0 and 7 (Sec. 3.3.2)
    seg = oracle.zigzag_segments(4)
    assert seg[0] == (0, 7)
    assert sorted(s for pair in seg for s in pair) == list(range(8))
    # balanced causal work: segment s needs s+1 key segments, so each device gets 2N+1 units
    assert all((a + 1) + (b + 1) == 9 for a, b in seg)


# ---------------------------------------------------------------- other step orders (Sec. 2.1, 3.3.2, 3.3.3)
def _causal_pairs(n):
    return [(c, j) for c in range(n) for j in range(c + 1)]


def test_other_orders_cover_every_needed_pair_once():
    for n in (1, 2, 4, 8):
        assert sorted(oracle.ring_attention_order(n, False)) == [(c, j) for c in range(n) for j in range(n)]
        assert sorted(oracle.ring_attention_order(n, True)) == _causal_pairs(n)
        assert sorted(oracle.zigzag_order(n)) == _causal_pairs(2 * n)
        for per_node in (d for d in (1, 2, 4, 8) if n % d == 0):
            assert sorted(oracle.hybrid_order(n // per_node, per_node, False)) == [(c, j) for c in range(n) for j in range(n)]
            assert sorted(oracle.hybrid_order(n // per_node, per_node, True)) == _causal_pairs(n)
    # Ring Attention: Query chunk j meets K/V chunks j, j-1, j-2, ... (the K/V ring runs the other way)
    assert [kv for q, kv in oracle.ring_attention_order(4, False) if q == 1] == [1, 0, 3, 2]


def test_orders_cover_pairs_for_every_small_device_count():
    for n in range(1, 13):
        full = [(c, j) for c in range(n) for j in range(n)]
        assert sorted((c, j) for _, j, c in oracle.ring_schedule(n, False)) == full
        assert sorted(oracle.ring_attention_order(n, False)) == full
        assert sorted(oracle.zigzag_order(n)) == _causal_pairs(2 * n)
        assert len(oracle.zigzag_order(n)) == n * (2 * n + 1)
        for per_node in (d for d in range(1, n + 1) if n % d == 0):
            assert sorted(oracle.hybrid_order(n // per_node, per_node, False)) == full
            assert sorted(oracle.hybrid_order(n // per_node, per_node, True)) == _causal_pairs(n)
        # every device of the zigzag partition owns the same amount of causal work: 2N + 1 segment pairs
        for a, b in oracle.zigzag_segments(n):
            assert (a + 1) + (b + 1) == 2 * n + 1


def test_hybrid_degenerates_to_its_two_ingredients():
    for causal in (False, True):
        # one node: plain Algorithm 1; one device per node: plain Ring Attention
        assert oracle.hybrid_order(1, 8, causal) == [(c, j) for _, j, c in oracle.ring_schedule(8, causal)]
        assert oracle.hybrid_order(8, 1, causal) == oracle.ring_attention_order(8, causal)
    # two nodes of four (the paper's figure): in the first outer step a node only touches its own K/V
    first = oracle.hybrid_order(2, 4, False)[:32]
    assert all((q // 4) == (kv // 4) for q, kv in first)
    assert all((q // 4) != (kv // 4) for q, kv in oracle.hybrid_order(2, 4, False)[32:])


def test_zigzag_balances_causal_work_and_releases_queries():
    n = 4
    steps = oracle.zigzag_steps(n)
    work = {}
    for i, j, qs, ks in steps:                      # a full segment pair is 1 unit, a diagonal one 1/2
        work[(i, j)] = work.get((i, j), 0.0) + (0.5 if qs == ks else 1.0)
    assert set(work) == {(i, j) for i in range(n) for j in range(n)} and set(work.values()) == {2.0}
    # contiguous chunks, by contrast, leave device loads between 1/2 and N - 1/2 units
    cont = {}
    for i, j, c in oracle.ring_schedule(n, True):
        cont[j] = cont.get(j, 0.0) + (0.5 if j == c else 1.0)
    assert min(cont.values()) == 0.5 and max(cont.values()) == n - 0.5
    # segment 0's Query is finished after iteration 0 (Sec. 3.3.2: it need not be sent on)
    assert {i for i, _, qs, _ in steps if qs == 0} == {0}
    # after iteration 0 a device either uses both Query segments on its first K/V segment or the
    # late Query segment on both K/V segments
    for i in range(1, n):
        for j in range(n):
            qs_ks = [(qs, ks) for ii, jj, qs, ks in steps if (ii, jj) == (i, j)]
            c = (j - i) % n
            expect = [(c, j), (2 * n - 1 - c, j)] if j < c else [(2 * n - 1 - c, j), (2 * n - 1 - c, 2 * n - 1 - j)]
            assert qs_ks == expect


@pytest.mark.parametrize("causal", [False, True])
def test_every_order_reaches_unchunked_attention(causal):
    B, Hq, Hkv, S, D = 1, 2, 1, 32, 8
    q, k, v = _rand((B, Hq, S, D), 71), _rand((B, Hkv, S, D), 72), _rand((B, Hkv, S, D), 73)
    ref_o, ref_l = oracle.attention_full(q, k, v, 0.3, causal=causal)
    orders = {"ring": (8, oracle.ring_attention_order(8, causal)), "hybrid": (8, oracle.hybrid_order(2, 4, causal))}
    if causal:
        orders["zigzag"] = (8, oracle.zigzag_order(4))
    for name, (n_seg, order) in orders.items():
        o, l = oracle.ring_attention(q, k, v, n_seg, causal, 0.3, order=order)
        assert np.allclose(o, ref_o, atol=1e-12, rtol=0), name
        assert np.allclose(l, ref_l, atol=1e-12, rtol=0), name
