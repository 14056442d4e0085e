"""Property tests of the oracle (hypothesis): invariants the formulation fixes, on random small problems."""
import numpy as np
import scipy.special
from hypothesis import given, settings, strategies as st

import oracle

SETTINGS = dict(max_examples=30, deadline=None, derandomize=True)


def _problem(seed, B, Hkv, G, S, D, std):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, Hkv * G, S, D)) * std
    k = rng.standard_normal((B, Hkv, S, D)) * std
    v = rng.standard_normal((B, Hkv, S, D))
    return q, k, v


shapes = st.tuples(st.integers(0, 2 ** 31 - 1), st.integers(1, 2), st.integers(1, 2), st.sampled_from([1, 2, 4]),
                   st.sampled_from([4, 6, 8, 12, 24]), st.sampled_from([2, 4, 8]), st.sampled_from([0.3, 1.0, 3.0]))


@settings(**SETTINGS)
@given(shapes, st.booleans(), st.floats(0.05, 1.5))
def test_rows_of_the_softmax_sum_to_one_and_lse_is_logsumexp(shape, causal, scale):
    q, k, v = _problem(*shape)
    out, lse = oracle.attention_full(q, k, v, scale, causal)
    S = q.shape[2]
    G = q.shape[1] // k.shape[1]
    for h in range(q.shape[1]):
        w = oracle.softmax_weights(q[0, h], k[0, h // G], scale, causal)
        assert np.allclose(w.sum(axis=1), 1.0, atol=1e-12)
        assert np.allclose(w @ v[0, h // G], out[0, h], atol=1e-12)
        s = scale * q[0, h] @ k[0, h // G].T
        if causal:
            s = np.where(np.tril(np.ones((S, S), dtype=bool)), s, -np.inf)
        assert np.allclose(scipy.special.logsumexp(s, axis=1), lse[0, h], atol=1e-12)


@settings(**SETTINGS)
@given(shapes, st.booleans(), st.floats(0.05, 1.5), st.integers(0, 2 ** 31 - 1))
def test_any_chunk_count_and_any_step_order_reach_unchunked_attention(shape, causal, scale, order_seed):
    q, k, v = _problem(*shape)
    S = q.shape[2]
    ref_o, ref_l = oracle.attention_full(q, k, v, scale, causal)
    for n in (d for d in (1, 2, 3, 4, S) if S % d == 0):
        o, l = oracle.ring_attention(q, k, v, n, causal, scale)
        assert np.allclose(o, ref_o, atol=1e-11) and np.allclose(l, ref_l, atol=1e-11)
        order = [(c, j) for _, j, c in oracle.ring_schedule(n, causal)]
        np.random.default_rng(order_seed).shuffle(order)
        o, l = oracle.ring_attention(q, k, v, n, causal, scale, order=order)
        assert np.allclose(o, ref_o, atol=1e-11) and np.allclose(l, ref_l, atol=1e-11)


@settings(**SETTINGS)
@given(st.integers(0, 2 ** 31 - 1), st.integers(1, 6), st.integers(1, 5), st.integers(1, 6))
def test_merge_is_order_free_and_matches_the_nary_definition(seed, n, rows, D):
    rng = np.random.default_rng(seed)
    outs = [rng.standard_normal((1, 1, rows, D)) for _ in range(n)]
    lses = [rng.uniform(-30, 30, (1, 1, rows)) for _ in range(n)]
    for l in lses:
        l[rng.random(l.shape) < 0.2] = -np.inf                 # empty partial rows
    ref_o, ref_l = oracle.merge_nary([np.where(np.isneginf(l)[..., None], 0.0, o) for o, l in zip(outs, lses)], lses)
    for perm in (range(n), reversed(range(n)), rng.permutation(n)):
        acc_o, acc_l = np.zeros((1, 1, rows, D)), np.full((1, 1, rows), -np.inf)
        for i in perm:
            acc_o, acc_l = oracle.merge_pair(acc_o, acc_l, np.where(np.isneginf(lses[i])[..., None], 0.0, outs[i]), lses[i])
        assert np.allclose(acc_o, ref_o, atol=1e-12) and np.allclose(acc_l, ref_l, atol=1e-12, equal_nan=False)
