"""The seeded input generator: determinism, distribution, storage rounding (no GPU)."""
import numpy as np

import blr_inputs as bi


def test_deterministic_and_streams_differ():
    a = bi.gaussian(1, bi.TID_X, (7, 9), 1.0, "f32")
    b = bi.gaussian(1, bi.TID_X, (7, 9), 1.0, "f32")
    c = bi.gaussian(1, bi.TID_R, (7, 9), 1.0, "f32")
    d = bi.gaussian(2, bi.TID_X, (7, 9), 1.0, "f32")
    np.testing.assert_array_equal(a.bits, b.bits)
    assert not np.array_equal(a.bits, c.bits) and not np.array_equal(a.bits, d.bits)


def test_moments():
    x = bi.standard_normal(3, 1, np.arange(400000))
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01
    assert abs((x ** 3).mean()) < 0.03 and abs((x ** 4).mean() - 3.0) < 0.06
    assert np.isfinite(x).all()


def test_bf16_rounding_is_nearest_even():
    # 1 + 2^-8 lies exactly between bf16 neighbours 1 and 1 + 2^-7: ties go to the even mantissa
    v = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7, 1.0 + 3 * 2.0 ** -8, -2.5, 0.0, 3.0e-3])
    bits = bi.round_to_bf16_bits(v)
    back = bi.bf16_bits_to_f64(bits)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.0 + 2.0 ** -7 and back[3] == 1.0 + 2.0 ** -6
    assert back[4] == -2.5 and back[5] == 0.0
    assert abs(back[6] - 3.0e-3) <= 3.0e-3 * 2.0 ** -8
    t = bi.gaussian(5, 1, (1000,), 1.0, "bf16")
    assert np.all(np.abs(t.f64 - bi.standard_normal(5, 1, np.arange(1000))) <= np.abs(t.f64) * 2.0 ** -8 + 1e-40)
    np.testing.assert_array_equal(bi.round_to_bf16_bits(t.f64), t.bits)   # stored values are fixed points


def test_scales_of_config_layers():
    lay = bi.make_layer(bi.CONFIGS["C0"])
    assert abs(lay.R.f64.std() * 8 - 1) < 0.05 and abs(lay.L.f64.std() * 8 - 1) < 0.05
    lay = bi.blast_layer(64, 64, 4, 16, "bf16")
    assert abs(lay.S.f64.std() * 4 - 1) < 0.2
