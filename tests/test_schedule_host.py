"""Host logic of the ring entry points, checked without a GPU: the step lists the library will run
(tr_schedule_steps) against the oracle's enumerations of the same schedules, and the invariants of
the grouping of steps into launches."""
import pytest

import oracle


@pytest.fixture(scope="module")
def tr():
    from paper_2412_20501_amd.build import ensure_built
    ensure_built()
    import paper_2412_20501_amd as m
    return m


def _pairs(steps):
    return [(q, k) for q, k, _ in steps]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("n", [1, 2, 3, 4, 8, 16])
def test_step_order_matches_the_oracle(tr, n, causal):
    assert _pairs(tr.tr_schedule_steps(tr.TR_SCHED_TOKENRING, n, causal)) == [(c, j) for _, j, c in oracle.ring_schedule(n, causal)]
    assert _pairs(tr.tr_schedule_steps(tr.TR_SCHED_RING_ATTENTION, n, causal)) == oracle.ring_attention_order(n, causal)
    for per_node in (d for d in (1, 2, 4, 8) if n % d == 0):
        got = _pairs(tr.tr_schedule_steps(tr.TR_SCHED_HYBRID, n, causal, per_node))
        assert got == oracle.hybrid_order(n // per_node, per_node, causal)


@pytest.mark.parametrize("n", [1, 2, 4, 5, 8])
def test_zigzag_steps_match_the_oracle_per_iteration_and_per_query_segment(tr, n):
    got = _pairs(tr.tr_schedule_steps(tr.TR_SCHED_ZIGZAG, n, True))
    ref = oracle.zigzag_steps(n)
    assert sorted(got) == sorted((qs, ks) for _, _, qs, ks in ref) and len(got) == n * (2 * n + 1)
    # iteration by iteration the same set of pairs (inside an iteration the devices run concurrently,
    # so their relative order is free) ...
    pos = 0
    for i in range(n):
        want = sorted((qs, ks) for ii, _, qs, ks in ref if ii == i)
        assert sorted(got[pos:pos + len(want)]) == want
        pos += len(want)
    # ... and every Query segment receives its blocks in the oracle's order
    for seg in range(2 * n):
        assert [ks for qs, ks in got if qs == seg] == [ks for _, _, qs, ks in ref if qs == seg]


@pytest.mark.parametrize("sched,n,inner,causal", [(0, 8, 1, True), (0, 16, 1, True), (0, 8, 1, False), (0, 40, 1, False), (1, 8, 1, True),
                                                  (2, 8, 1, True), (2, 4, 1, True), (3, 8, 4, True), (3, 12, 3, False)])
def test_launch_grouping_invariants(tr, sched, n, inner, causal):
    steps = tr.tr_schedule_steps(sched, n, causal, inner)
    launches = [g for _, _, g in steps]
    assert launches == sorted(launches) and launches[0] == 0 and set(launches) == set(range(launches[-1] + 1))
    seen = set()
    for g in range(launches[-1] + 1):
        in_g = [(q, k) for q, k, gg in steps if gg == g]
        if sched == 2:
            # zigzag: a step over the device's K/V pair is listed as two adjacent entries (q, k), (q, 2n-1-k)
            fused = [a for a, b in zip(in_g, in_g[1:]) if a[0] == b[0]]
            assert all((q, 2 * n - 1 - k) == in_g[in_g.index((q, k)) + 1] and k < n <= q for q, k in fused)
            in_g = [e for e in in_g if not any(e == (q, 2 * n - 1 - k) for q, k in fused)]
            assert len(fused) == n - g                                          # iteration g: the devices whose K/V pair does not lie before the Query pair
        qsegs = [q for q, _ in in_g]
        assert 1 <= len(qsegs) <= 32 and len(set(qsegs)) == len(qsegs)          # independent steps only
        kinds = {q in seen for q in qsegs}
        assert len(kinds) == 1                                                  # all first blocks, or all later blocks
        seen.update(qsegs)
    if sched == 0 and causal:
        assert launches[-1] + 1 == n                      # Algorithm 1 on contiguous causal chunks: one launch per iteration or fewer
    if sched == 2:
        assert launches[-1] + 1 == n                      # zigzag: one launch per iteration
    if sched == 0 and not causal and n <= 32:
        assert launches[-1] + 1 == n                      # every iteration is one launch


def test_schedule_argument_errors(tr):
    lib = tr.raw_lib()
    assert lib.tr_schedule_steps(9, 4, 1, 1, None, 0) == -1
    assert lib.tr_schedule_steps(tr.TR_SCHED_ZIGZAG, 4, 1, 0, None, 0) == -1 and b"zigzag" in lib.tr_last_error()
    assert lib.tr_schedule_steps(tr.TR_SCHED_HYBRID, 6, 4, 1, None, 0) == -1
    assert lib.tr_schedule_steps(tr.TR_SCHED_TOKENRING, 0, 1, 1, None, 0) == -1
    assert lib.tr_schedule_steps(tr.TR_SCHED_TOKENRING, 8, 1, 1, None, 0) == 36
    assert lib.tr_schedule_steps(tr.TR_SCHED_TOKENRING, 16, 1, 1, None, 0) == 136
