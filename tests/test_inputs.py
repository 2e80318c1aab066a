"""Checks of the seeded input generator (host logic only)."""
import numpy as np
import pytest

import mst_inputs as mi


def test_bf16_round_to_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -7, -2.5, 0.0, 3.0e38], dtype=np.float32)
    bits = mi.f32_to_bf16_bits(x)
    back = mi.bf16_bits_to_f32(bits)
    # ties go to the even mantissa: 1 + 2^-8 -> 1 ; 1 + 3*2^-8 -> 1 + 2^-6
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == np.float32(1.0 + 2 ** -6)
    assert back[3] == np.float32(1.0 + 2 ** -7) and back[4] == -2.5 and back[5] == 0.0
    torch = pytest.importorskip("torch")
    r = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    t = torch.from_numpy(r).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(mi.f32_to_bf16_bits(r), t)


def test_config_shapes_and_ignored_counts():
    exp = {1: (512, 256, 4096, 4, 480), 2: (8192, 4096, 128256, 8, 8110), 3: (32768, 4096, 128256, 32, 32440),
           4: (16384, 3584, 256000, 16, 16056), 5: (131072, 4096, 32768, 64, 124518)}
    for i, (S, d, V, M, nv) in exp.items():
        cfg = mi.CONFIGS[i]
        assert (cfg.S, cfg.d, cfg.V, cfg.M) == (S, d, V, M)
        y = mi.make_labels(cfg)
        assert y.dtype == np.int32 and y.shape == (S,)
        valid = y != mi.IGNORE_INDEX
        assert int(valid.sum()) == nv
        assert y[valid].min() >= 0 and y[valid].max() < V


def test_config1_tensors_are_seeded_and_distributed_as_stated():
    a, b = mi.make_inputs(1), mi.make_inputs(1)
    np.testing.assert_array_equal(a.H_bits, b.H_bits)
    np.testing.assert_array_equal(a.W_bits, b.W_bits)
    np.testing.assert_array_equal(a.labels, b.labels)
    assert (a.labels[15::16] == -100).all() and (a.labels[0:15] != -100).all()
    assert a.H_f64().std() == pytest.approx(1.0, rel=0.02)
    assert a.W_f64().std() == pytest.approx(0.02, rel=0.02)


def test_zipf_labels_are_heavy_tailed():
    y = mi.make_labels(mi.CONFIGS[3])
    y = y[y != -100]
    counts = np.bincount(y, minlength=128256)
    top = np.sort(counts)[::-1]
    # Zipf(1.1) over 128256 ranks: rank 1 carries ~ 1 / H_{V,1.1} ~ 14 % of the mass
    assert 0.10 < top[0] / len(y) < 0.18
    assert top[0] > 1.8 * top[1] * 0.8
