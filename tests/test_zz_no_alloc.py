"""tr_ring_attn_noalloc (the two-kernel ring form with the block workspace inside the library)
against tr_ring_attn with a caller workspace (bitwise: same kernels, same order) and against
the fp64 oracle, on two calls in a row, the second with a smaller input: the library's
scratch array keeps the first call's contents, which must not leak into the second."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import bits_to_dev, f64, max_abs, rand_bits, to_np

pytestmark = pytest.mark.gpu
OUT_TOL, LSE_TOL = 1e-2, 1e-3


def _run_both(lib, shape, n_chunks, causal, seed):
    B, Hq, Hkv, S, D = shape
    qb, kb, vb = rand_bits((B, Hq, S, D), seed), rand_bits((B, Hkv, S, D), seed + 1), rand_bits((B, Hkv, S, D), seed + 2)
    q, k, v = bits_to_dev(qb), bits_to_dev(kb), bits_to_dev(vb)
    nan = float("nan")
    out_ws = torch.full((B, Hq, S, D), nan, dtype=torch.float32, device="cuda"); lse_ws = torch.full((B, Hq, S), nan, dtype=torch.float32, device="cuda")
    out_na = torch.full((B, Hq, S, D), nan, dtype=torch.float32, device="cuda"); lse_na = torch.full((B, Hq, S), nan, dtype=torch.float32, device="cuda")
    ws = torch.empty(max(256, lib.tr_ring_attn_workspace_bytes(q, n_chunks)), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    lib.tr_ring_attn_noalloc(q, k, v, n_chunks, causal, out_na, lse_na)            # scale 0 -> 1/sqrt(D)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before                                  # nothing was taken from torch's pool either
    lib.tr_ring_attn(q, k, v, n_chunks, causal, out_ws, lse_ws, 0.0, ws)
    torch.cuda.synchronize()
    assert torch.equal(out_na, out_ws) and torch.equal(lse_na, lse_ws), "differs from tr_ring_attn with a workspace"
    ref_o, ref_l = oracle.attention_full(f64(qb), f64(kb), f64(vb), 1.0 / np.sqrt(D), causal)
    d_o, d_l = max_abs(to_np(out_na), ref_o), max_abs(to_np(lse_na), ref_l)
    assert d_o <= OUT_TOL and d_l <= LSE_TOL, (d_o, d_l)
    return d_o, d_l


def test_noalloc_two_calls_second_smaller(lib):
    big = _run_both(lib, (1, 8, 4, 1536, 128), 3, True, seed=71)      # chunk 512: several query tiles, GQA, causal
    small = _run_both(lib, (2, 2, 2, 200, 64), 4, False, seed=81)     # chunk 50: ragged tiles, D = 64, non-causal
    again = _run_both(lib, (1, 8, 4, 1536, 128), 3, True, seed=71)    # and the larger one once more: same result
    assert again == big
    print(f"noalloc: big {big}, small {small}")


def test_noalloc_rejects_what_does_not_fit(lib):
    # one block result of B1 H32 C4096 D128 is 64 MiB: far beyond the built-in scratch
    q = torch.empty((1, 32, 8192, 128), dtype=torch.bfloat16, device="cuda")
    out = torch.empty((1, 32, 8192, 128), dtype=torch.float32, device="cuda"); lse = torch.empty((1, 32, 8192), dtype=torch.float32, device="cuda")
    with pytest.raises(lib.TokenRingError) as e:
        lib.tr_ring_attn_noalloc(q, q, q, 2, True, out, lse)
    assert e.value.status == 7 and "scratch" in str(e.value)
