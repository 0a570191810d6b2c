"""The seeded input generator: determinism, rounding, distribution and the outlier recipe (CPU only)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2312_11918_amd import workloads


def test_config_table_matches_the_five_workloads():
    shapes = {i: (w.B, w.H, w.N, w.d, w.dtype) for i, w in workloads.CONFIGS.items()}
    assert shapes == {1: (1, 2, 256, 64, "fp16"), 2: (32, 16, 512, 64, "fp16"), 3: (8, 16, 2048, 128, "fp16"),
                      4: (2, 16, 8192, 128, "bf16"), 5: (1, 32, 16384, 64, "fp16")}
    assert workloads.CONFIGS[3].flops == pytest.approx(2.749e11, rel=1e-3)
    assert workloads.CONFIGS[3].scale == pytest.approx(128 ** -0.5, rel=1e-7)


def test_generator_is_deterministic_and_ordered():
    a = workloads.make_qkv(1, 64, 2, 16, "fp16", seed=5)
    b = workloads.make_qkv(1, 64, 2, 16, "fp16", seed=5)
    c = workloads.make_qkv(1, 64, 2, 16, "fp16", seed=6)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    assert not np.array_equal(a[0], c[0])
    # Q is the first draw of the stream
    ref = np.random.Generator(np.random.PCG64(5)).standard_normal((1, 64, 2, 16), dtype=np.float32)
    assert np.array_equal(a[0], ref.astype(np.float16).view(np.uint16))


def test_bf16_rounding_is_nearest_even():
    r = np.random.Generator(np.random.PCG64(1))
    x = np.concatenate([r.standard_normal(20000, dtype=np.float32) * 8,
                        np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 0.0, 3.0e-39], dtype=np.float32)])
    bits = workloads.round_to_bits(x, "bf16")
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    # ties: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 -> 1 + 2^-6
    assert workloads.round_to_bits(np.array([1.00390625, 1.01171875], np.float32), "bf16").tolist() == [0x3F80, 0x3F82]


def test_fp16_bits_roundtrip_through_oracle_widen():
    x = np.array([0.1, -2.5, 65504.0, 1e-8], dtype=np.float32)
    assert np.array_equal(oracle.widen(workloads.round_to_bits(x, "fp16"), "fp16"), x.astype(np.float16).astype(np.float64))


def test_distribution_is_standard_normal():
    q, k, v = workloads.make_qkv(2, 512, 4, 64, "fp16", seed=7)
    for bits in (q, k, v):
        x = oracle.widen(bits, "fp16")
        assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01


def test_outlier_rows_recipe():
    N, H = 1000, 3
    q, k, v = workloads.make_qkv(1, N, H, 32, "fp16", seed=9, k_outlier_frac=0.01, k_outlier_gain=8.0)
    q0, k0, v0 = workloads.make_qkv(1, N, H, 32, "fp16", seed=9)
    assert np.array_equal(q, q0) and np.array_equal(v, v0)
    kw, kw0 = oracle.widen(k, "fp16"), oracle.widen(k0, "fp16")
    for h in range(H):
        changed = np.where(np.any(kw[0, :, h] != kw0[0, :, h], axis=1))[0]
        assert len(changed) == 10                                # round(0.01 * 1000) distinct rows per head
        np.testing.assert_allclose(kw[0, changed, h], 8.0 * kw0[0, changed, h], rtol=2 ** -10)
    rms = np.sqrt((kw[0] ** 2).mean())
    assert 1.2 < rms < 1.4                                        # sqrt(0.99 + 0.01*64) = 1.277
