"""tr_time_next_kernel: the armed events bracket exactly one kernel and do not change its result."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_events_time_one_kernel_and_leave_results_alone(lib):
    tr = lib
    g = torch.Generator(device="cuda").manual_seed(7)
    B, H, S, D = 1, 4, 1000, 128
    acc = torch.randn((B, H, S, D), device="cuda", generator=g)
    accl = torch.randn((B, H, S), device="cuda", generator=g)
    blk = torch.randn((B, H, S, D), device="cuda", generator=g)
    bl = torch.randn((B, H, S), device="cuda", generator=g)
    ref_o, ref_l = acc.clone(), accl.clone()
    tr.tr_merge(ref_o, ref_l, blk, bl)

    k0, k1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    w0, w1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    o, l = acc.clone(), accl.clone()
    torch.cuda.synchronize()
    w0.record()
    tr.tr_time_next_kernel(k0, k1)
    tr.tr_merge(o, l, blk, bl)
    w1.record()
    torch.cuda.synchronize()
    assert torch.equal(o, ref_o) and torch.equal(l, ref_l)
    inner, outer = k0.elapsed_time(k1), w0.elapsed_time(w1)
    assert 0.0 < inner <= outer + 1e-3

    # the arming is consumed by that launch: a later call leaves the events untouched
    before = k0.elapsed_time(k1)
    tr.tr_merge(o, l, blk, bl)
    torch.cuda.synchronize()
    assert k0.elapsed_time(k1) == before
