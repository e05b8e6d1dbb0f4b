"""The seeded input generators (no arithmetic of the method): determinism, formats, and the
residual-stream stand-in that feeds the predictor accuracy figures."""
import numpy as np

import synth_inputs as si


def test_layers_are_reproducible_and_parts_can_be_drawn_alone():
    cfg = si.small_config(T=40, d=64, E=4, k=2, F=128)
    a = si.make_layer(cfg)
    b = si.make_layer(cfg, parts=("w2", "x"))
    assert np.array_equal(a["x"], b["x"]) and np.array_equal(a["w2"], b["w2"])
    w1, w3, w2 = si.expert_weights(cfg, 3)
    assert np.array_equal(w1, a["w1"][3]) and np.array_equal(w3, a["w3"][3]) and np.array_equal(w2, a["w2"][3])
    other = si.make_layer(si.small_config(T=40, d=64, E=4, k=2, F=128, seed=8), parts=("x",))
    assert not np.array_equal(a["x"], other["x"])


def test_bf16_rounding_is_nearest_even_and_widening_is_exact():
    vals = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -9, -2.5, 0.0], np.float32)
    bits = si.f32_to_bf16_bits(vals)
    back = si.bf16_bits_to_f32(bits)
    # an ulp at 1.0 is 2^-7; ties go to the even mantissa: 1 + 2^-8 -> 1, 1 + 3*2^-8 -> 1 + 2^-6
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == np.float32(1.0 + 2.0 ** -6)
    assert back[3] == 1.0 and back[4] == -2.5 and back[5] == 0.0
    assert np.array_equal(si.f32_to_bf16_bits(back), bits)          # idempotent


def test_residual_step_is_seeded_additive_noise_in_the_layer_dtype():
    for dtype in (si.BF16, si.F32):
        cfg = si.small_config(T=200, d=128, dtype=dtype, x_std=0.5)
        x = si.make_layer(cfg, parts=("x",))["x"]
        same = si.residual_step(cfg, x, 0.0)
        assert same.dtype == x.dtype and np.array_equal(same, x)
        a, b = si.residual_step(cfg, x, 0.25), si.residual_step(cfg, x, 0.25)
        assert np.array_equal(a, b)                                  # seeded
        assert not np.array_equal(a, si.residual_step(cfg, x, 0.25, step=2))
        f = (lambda v: v) if dtype == si.F32 else si.bf16_bits_to_f32
        delta = f(a).astype(np.float64) - f(x).astype(np.float64)
        # eps * x_std = 0.125: the added noise has that scale (bf16 rounding adds well under 1 %)
        assert abs(delta.std() / 0.125 - 1.0) < 0.03 and abs(delta.mean()) < 0.005
