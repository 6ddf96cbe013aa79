"""The seeded input recipe: determinism, shapes, distributions, bf16 rounding."""
import numpy as np
import pytest

import grkan_inputs as gi


def test_config_shapes_match_the_kat_variants():
    assert gi.CONFIGS["tiny"].rows == 788
    for name, d1, d2 in (("kat_t", 192, 768), ("kat_s", 384, 1536), ("kat_b", 768, 3072)):
        cfg = gi.CONFIGS[name]
        assert cfg.rows == 128 * 197
        assert cfg.D("x1") == d1 and cfg.D("x2") == d2 == 4 * d1
    assert gi.CONFIGS["stress"].rows == 256 * 197 and gi.CONFIGS["stress"].D("x") == 3072


def test_cases_are_reproducible_and_prefix_stable():
    a = gi.make_case("kat_t", "x1", rows=64)
    b = gi.make_case("kat_t", "x1", rows=64)
    c = gi.make_case("kat_t", "x1", rows=16)
    for k in ("x", "dy", "A", "B"):
        assert np.array_equal(a[k], b[k])
    assert np.array_equal(a["x"][:16], c["x"]) and np.array_equal(a["dy"][:16], c["dy"])
    s64 = gi.make_case("stress", rows=8)
    s16 = gi.make_case("stress", rows=2)
    assert np.array_equal(s64["x"][:2], s16["x"])
    # different tensors of one config are different streams
    x2 = gi.make_case("kat_t", "x2", rows=16)
    assert not np.array_equal(x2["x"][:, :192], c["x"])


def test_coefficient_recipe():
    A, B = gi.coefficients(gi.CONFIGS["tiny"])
    assert A.shape == (8, 6) and B.shape == (8, 4) and A.dtype == np.float32
    assert np.all(np.abs(A) <= 1.0 / (np.arange(6) + 1.0)) and np.all(np.abs(B) <= 0.5)
    A64, B64 = gi.coefficients(gi.CONFIGS["stress"], G=64)
    assert A64.shape == (64, 6) and B64.shape == (64, 4)


def test_distributions():
    c = gi.make_case("kat_t", "x2", rows=2000)
    assert abs(c["x"].mean()) < 5e-3 and abs(c["x"].std() - 1) < 5e-3
    assert abs(c["dy"].std() - 0.01) < 1e-4
    s = gi.make_case("stress", rows=400)
    # Student-t(3): variance 3, heavy tails
    assert np.abs(s["x"]).max() > 20
    assert 0.60 < np.mean(np.abs(s["x"]) < 1.0) < 0.62  # P(|t3| < 1) = 0.609


def test_bf16_rounding_is_nearest_even():
    f = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -7, -2.5, 3.1415927, 1e-20], dtype=np.float32)
    bits = gi.round_to_bf16_bits(f)
    back = gi.bf16_bits_to_f32(bits)
    # ties: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> even mantissa (1.0);
    #       1 + 3*2^-8 is halfway between 1+2^-7 and 1+2^-6 -> 1 + 2^-6
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == np.float32(1.0 + 2 ** -6) and back[3] == np.float32(1 + 2 ** -7)
    assert back[4] == -2.5
    assert abs(back[5] - f[5]) <= 2 ** -8 * abs(f[5])
    assert np.all(np.abs(back - f) <= np.abs(f) * 2.0 ** -8)
    c = gi.make_case("kat_b", "x1", dtype="bf16", rows=4)
    assert c["x_bits"].dtype == np.uint16
    assert np.array_equal(gi.bf16_bits_to_f32(c["x_bits"]), c["x"])
    assert np.array_equal(gi.round_to_bf16_bits(c["x"]), c["x_bits"])


def test_bad_requests():
    with pytest.raises(ValueError):
        gi.make_case("kat_b", "x3")
    with pytest.raises(ValueError):
        gi.make_case("tiny", G=7)
    with pytest.raises(ValueError):
        gi.make_case("tiny", dtype="f64")


def test_f16_rounding_is_nearest_even_and_exactly_widened():
    # 1 + 2^-11 lies halfway between 1 and the next binary16 value 1 + 2^-10: ties go to the even one
    f = np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -11 + 2.0 ** -20, 65504.0, 2.0 ** -24],
                 dtype=np.float32)
    back = gi.f16_bits_to_f32(gi.round_to_f16_bits(f))
    assert back.tolist() == [1.0, 1.0 + 2.0 ** -9, 1.0 + 2.0 ** -10, 65504.0, 2.0 ** -24]
    c = gi.make_case("kat_b", "x1", dtype="f16", rows=4)
    assert c["x_bits"].dtype == np.uint16
    assert np.array_equal(gi.f16_bits_to_f32(c["x_bits"]), c["x"])
    assert np.array_equal(gi.round_to_f16_bits(c["x"]), c["x_bits"])
    # same draws as the float32 case, rounded once
    c32 = gi.make_case("kat_b", "x1", dtype="f32", rows=4)
    assert np.max(np.abs(c["x"] - c32["x"]) / np.maximum(np.abs(c32["x"]), 2.0 ** -14)) <= 2.0 ** -11


def test_other_degrees_reuse_the_coefficient_streams():
    cfg = gi.CONFIGS["tiny"]
    A54, B54 = gi.coefficients(cfg)
    A32, B32 = gi.coefficients(cfg, m=3, n=2)
    A76, B76 = gi.coefficients(cfg, m=7, n=6)
    assert A32.shape == (8, 4) and B32.shape == (8, 2) and A76.shape == (8, 8) and B76.shape == (8, 6)
    assert np.all(np.abs(A76) <= 1.0 / (np.arange(8) + 1.0)) and np.all(np.abs(B76) <= 0.5)
    c = gi.make_case("tiny", m=7, n=6)
    assert (c["m"], c["n"]) == (7, 6) and np.array_equal(c["A"], A76)
    # x and dy do not depend on the degrees
    assert np.array_equal(c["x"], gi.make_case("tiny")["x"])
