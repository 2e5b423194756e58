"""The seeded input recipes: determinism, shapes and the value structure they promise."""
import numpy as np

import synthetic_inputs as si


def test_small_configs_are_deterministic_and_shaped():
    a = si.make("cfg1_act")
    b = si.make("cfg1_act")
    assert a.shape == (4, 64, 32, 32) and a.dtype == np.float32
    assert a.tobytes() == b.tobytes()
    assert 0.48 < float((a == 0).mean()) < 0.52 and a.min() == 0.0
    g = si.make("cfg2_grad")
    assert g.shape == (4, 64, 32, 32)
    assert 0.8e-3 < float(np.median(np.abs(g))) / 0.6745 < 1.2e-3
    assert float(np.abs(g).max()) > 0.05  # the 0.1 % outliers dominate the range
    assert si.as_nm(g) == (4, 65536)


def test_recipes_on_small_shapes():
    x = si.make_shape("relu_lognormal", (8, 16, 7, 7), 2)
    assert 0.55 < float((x == 0).mean()) < 0.65 and x.min() == 0.0
    y = si.make_shape("relu_lognormal_chgain", (8, 16, 7, 7), 3)
    ch_max = y.max(axis=(0, 2, 3))
    assert len(set(np.round(ch_max, 3).tolist())) > 8  # channels really differ in range
    t = si.make_shape("student_t3", (4, 33, 17), 5)
    assert t.shape == (4, 33, 17) and float(np.abs(t).max()) > 4.0
    assert si.CONFIGS["cfg4_act"][0] == (64, 256, 56, 56)
    assert si.CONFIGS["cfg5_hidden"][0] == (16, 509, 768)


def test_bf16_bits_round_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0], dtype=np.float32)
    # 1.00390625 = 1 + 2^-8 is a tie between 1.0 and 1.0078125 -> even (1.0);
    # 1.01171875 = 1 + 3*2^-8 is a tie -> even mantissa (1.015625)
    assert si.to_bf16_bits(x).tolist() == [0x3F80, 0x3F80, 0x3F82, 0xC020, 0x0000]
