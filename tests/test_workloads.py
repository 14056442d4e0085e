"""The seeded input generators: bf16 rounding, shapes, determinism (CPU only)."""
import numpy as np
import torch

import workloads as wl


def test_bf16_rounding_matches_torch_rne():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e38, -1e-30], dtype=np.float32)])
    bits = wl.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    back = wl.bf16_bits_to_f32(bits)
    assert np.array_equal(wl.f32_to_bf16_bits(back), bits)
    assert np.array_equal(wl.bf16_bits_to_f64(bits), back.astype(np.float64))
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(np.array([1.00390625], np.float32)))[0] == 1.0
    assert wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(np.array([1.01171875], np.float32)))[0] == 1.015625


def test_qkv_shapes_determinism_and_distribution():
    cfg = wl.CONFIGS["cfg1_small"]
    q, k, v = wl.make_qkv_bits(cfg)
    q2, k2, v2 = wl.make_qkv_bits(cfg)
    assert q.shape == (1, 2, 256, 64) and k.shape == v.shape == (1, 2, 256, 64) and q.dtype == np.uint16
    assert np.array_equal(q, q2) and np.array_equal(k, k2) and np.array_equal(v, v2)
    x = wl.bf16_bits_to_f64(np.concatenate([q.ravel(), k.ravel(), v.ravel()]))
    assert abs(x.mean()) < 0.02 and abs(x.std() - 1.0) < 0.02
    assert not np.array_equal(q, k)
    assert abs(cfg.scale - 0.125) < 1e-15 and cfg.chunk == 64


def test_config_table_matches_the_five_workloads():
    c = wl.CONFIGS
    assert (c["cfg2_block"].Hq, c["cfg2_block"].S, c["cfg2_block"].D) == (32, 4096, 128)
    assert (c["cfg3_ring"].S, c["cfg3_ring"].n_chunks, c["cfg3_ring"].chunk, c["cfg3_ring"].causal) == (32768, 8, 4096, True)
    assert (c["cfg5_gqa"].Hq, c["cfg5_gqa"].Hkv, c["cfg5_gqa"].S, c["cfg5_gqa"].chunk, c["cfg5_gqa"].std) == (32, 8, 131072, 8192, 0.5)
    m = c["cfg4_merge"]
    assert (m.H, m.S, m.D, m.n_partials) == (32, 32768, 128, 8)
    outs, lses = wl.make_merge_partials(m, S=64)
    assert len(outs) == 8 and outs[0].shape == (1, 32, 64, 128) and lses[0].shape == (1, 32, 64)
    assert outs[0].dtype == np.float32 and lses[0].dtype == np.float32
    allv = np.concatenate([l.ravel() for l in lses])
    assert allv.min() >= -5.0 and allv.max() <= 15.0 and abs(allv.mean() - 5.0) < 0.2


def test_sample_rows_cover_boundaries():
    rows = wl.sample_rows(32768, 4096, 64, seed=1)
    for r in (0, 1, 2, 4095, 4096, 4097, 28671, 28672, 28673, 32766, 32767):
        assert r in rows
    assert np.all(np.diff(rows) > 0) and rows.min() >= 0 and rows.max() < 32768
    assert np.array_equal(rows, wl.sample_rows(32768, 4096, 64, seed=1))
