"""The entry points only enqueue kernels on the caller's stream: they work on a non-default stream,
and a whole ring schedule can be captured into a HIP graph and replayed (no allocation, no
synchronisation, no memset inside the library)."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import bits_to_dev, f64, max_abs, rand_bits, to_np

pytestmark = pytest.mark.gpu


def _inputs(seed, B=1, Hq=4, Hkv=2, S=512, D=128):
    qb, kb, vb = rand_bits((B, Hq, S, D), seed), rand_bits((B, Hkv, S, D), seed + 1), rand_bits((B, Hkv, S, D), seed + 2)
    return (qb, kb, vb), (bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb))


def test_side_stream_gives_the_default_stream_result(lib):
    (qb, kb, vb), (q, k, v) = _inputs(60)
    out0 = torch.empty((1, 4, 512, 128), dtype=torch.float32, device="cuda"); lse0 = torch.empty((1, 4, 512), device="cuda")
    lib.tr_ring_attn(q, k, v, 4, True, out0, lse0, 0.0, None)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    out1 = torch.full_like(out0, float("nan")); lse1 = torch.full_like(lse0, float("nan"))
    side.wait_stream(torch.cuda.current_stream())
    lib.tr_ring_attn(q, k, v, 4, True, out1, lse1, 0.0, None, side)
    blk_o = torch.empty((1, 4, 512, 128), dtype=torch.float32, device="cuda"); blk_l = torch.empty((1, 4, 512), device="cuda")
    acc_o = torch.zeros_like(out0)
    acc_l = torch.full_like(lse0, float("-inf"))
    with torch.cuda.stream(side):
        lib.tr_block_attn(q, k, v, lib.TR_MASK_CAUSAL_DIAG, 1.0 / np.sqrt(128), blk_o, blk_l)   # binding default = current stream
        lib.tr_merge(acc_o, acc_l, blk_o, blk_l)
    side.synchronize()
    assert torch.equal(out0, out1) and torch.equal(lse0, lse1)
    ref_o, ref_l = oracle.attention_full(f64(qb), f64(kb), f64(vb), 1.0 / np.sqrt(128), True)
    assert max_abs(to_np(acc_o), ref_o) <= 1e-2 and max_abs(to_np(acc_l), ref_l) <= 1e-3


@pytest.mark.parametrize("fused", [True, False])
def test_ring_schedule_captured_in_a_graph_replays_exactly(lib, fused):
    (qb, kb, vb), (q, k, v) = _inputs(63)
    shape_o, shape_l = (1, 4, 512, 128), (1, 4, 512)
    ws = None if fused else torch.empty(lib.tr_ring_attn_workspace_bytes(q, 4), dtype=torch.uint8, device="cuda")
    eager_o = torch.empty(shape_o, dtype=torch.float32, device="cuda"); eager_l = torch.empty(shape_l, device="cuda")
    lib.tr_ring_attn(q, k, v, 4, True, eager_o, eager_l, 0.0, ws)      # also sets the kernels' LDS attribute before capture
    torch.cuda.synchronize()
    out = torch.zeros(shape_o, dtype=torch.float32, device="cuda"); lse = torch.zeros(shape_l, device="cuda")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lib.tr_ring_attn(q, k, v, 4, True, out, lse, 0.0, ws)
    for replay in range(3):
        out.fill_(float("nan")); lse.fill_(float("nan"))               # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager_o) and torch.equal(lse, eager_l), f"replay {replay}"
    # new inputs in the same buffers: the graph recomputes, it has not baked results in
    q2 = bits_to_dev(rand_bits((1, 4, 512, 128), 70))
    q.copy_(q2)
    lib.tr_ring_attn(q, k, v, 4, True, eager_o, eager_l, 0.0, ws)
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, eager_o) and torch.equal(lse, eager_l)


def test_zigzag_schedule_with_paired_segments_replays_from_a_graph(lib):
    """The zigzag order on 128-key segments (block steps over a device's K/V pair, steps of a launch sorted by length)
    captured once and replayed with eager work in between: every replay equals the eager result bitwise."""
    qb, kb, vb = rand_bits((1, 4, 1024, 128), 91), rand_bits((1, 2, 1024, 128), 92), rand_bits((1, 2, 1024, 128), 93)
    q, k, v = bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb)
    shape_o, shape_l = (1, 4, 1024, 128), (1, 4, 1024)
    eager_o = torch.empty(shape_o, dtype=torch.float32, device="cuda"); eager_l = torch.empty(shape_l, device="cuda")
    lib.tr_ring_attn_sched(q, k, v, 4, True, lib.TR_SCHED_ZIGZAG, eager_o, eager_l)
    torch.cuda.synchronize()
    ref_o, ref_l = oracle.attention_full(f64(qb), f64(kb), f64(vb), 1.0 / np.sqrt(128), True)
    assert max_abs(to_np(eager_o), ref_o) <= 1e-2 and max_abs(to_np(eager_l), ref_l) <= 1e-3
    out = torch.zeros(shape_o, dtype=torch.float32, device="cuda"); lse = torch.zeros(shape_l, device="cuda")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lib.tr_ring_attn_sched(q, k, v, 4, True, lib.TR_SCHED_ZIGZAG, out, lse)
    for replay in range(3):
        out.fill_(float("nan")); lse.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager_o) and torch.equal(lse, eager_l), f"replay {replay}"
