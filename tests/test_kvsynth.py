"""The input generators: determinism, shapes, and the structure the recipe promises."""
import numpy as np

import kvsynth
from kvsynth.generate import generate, sequence_duplicates


def test_units_are_reproducible_and_order_independent():
    cfg = kvsynth.get_config("mid").scaled(n_tokens=256, layers=2, kv_heads=2)
    K1, V1 = generate(cfg, workers=1)
    K2, V2 = generate(cfg, workers=4)
    assert np.array_equal(K1, K2) and np.array_equal(V1, V2)
    k, v = kvsynth.generate_unit(cfg, 0, 1, 1)
    assert np.array_equal(k, K1[0, 1, 1]) and np.array_equal(v, V1[0, 1, 1])
    assert K1.dtype == np.uint16 and K1.shape == (1, 2, 2, 256, 128)


def test_bf16_round_trip_and_rounding():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.1], dtype=np.float32)
    bits = kvsynth.f32_to_bf16_bits(x)
    back = kvsynth.bf16_bits_to_f32(bits)
    # 1.00390625 = 1 + 2^-8 is a tie -> even (1.0); 1.01171875 = 1 + 3*2^-8 -> 1 + 2^-6
    assert back.tolist()[:4] == [1.0, 1.0, 1.015625, -2.5]
    assert abs(back[4] - 0.1) <= 0.1 * 2.0 ** -8
    assert np.array_equal(kvsynth.f32_to_bf16_bits(back), bits)


def test_outliers_shared_by_heads_and_tensors():
    cfg = kvsynth.get_config("tiny")
    pos, mag = kvsynth.layer_outlier_positions(cfg, 0, 0)
    assert len(pos) == 10 and np.all(np.diff(pos) > 0) and np.all(mag == 3.0)
    K, V = generate(cfg)
    norms = np.linalg.norm(K[0, 0, 1].astype(np.float64), axis=1)
    assert set(np.argsort(-norms)[:10].tolist()) == set(pos.tolist())


def test_blocks_layout_and_duplicates():
    cfg = kvsynth.get_config("batch8_16k").scaled(batch=1, layers=1, kv_heads=1, n_tokens=2048,
                                                  block_len=240)
    assert cfg.visual_end == 64 + 8 * 240
    k, v = kvsynth.generate_unit(cfg, 0, 0, 0)
    x = kvsynth.bf16_bits_to_f32(k).astype(np.float64)
    src, dst = sequence_duplicates(cfg, 0)
    assert len(src) == 10 and np.array_equal(k[dst], k[src]) and np.array_equal(v[dst], v[src])
    text = np.r_[0:64, cfg.visual_end:2048]
    assert 0.8 < x[text].std() < 1.2
