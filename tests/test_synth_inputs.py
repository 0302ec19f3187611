"""The seeded input generator: reproducible, sliceable, N(0,1) to within sampling error, exact bf16."""
import numpy as np

import synth_inputs as si


def test_reproducible_and_sliceable():
    a = si.normal_bf16_bits(123, 2, 10000)
    b = si.normal_bf16_bits(123, 2, 10000, chunk=777)
    np.testing.assert_array_equal(a, b)
    c = si.normal_bf16_bits(123, 2, 100, offset=5000)
    np.testing.assert_array_equal(a[5000:5100], c)
    assert not np.array_equal(a, si.normal_bf16_bits(124, 2, 10000))
    assert not np.array_equal(a, si.normal_bf16_bits(123, 3, 10000))


def test_moments():
    x = si.bf16_bits_to_f64(si.normal_bf16_bits(99, 0, 1 << 20))
    assert abs(x.mean()) < 5e-3
    assert abs(x.std() - 1.0) < 5e-3
    assert abs((x ** 3).mean()) < 2e-2
    assert abs((x ** 4).mean() - 3.0) < 5e-2
    assert np.all(np.isfinite(x))


def test_bf16_rounding_is_nearest_even():
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: goes to even (1.0); 1 + 3*2^-8 goes up to 1 + 2^-6
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -7, -2.5, 0.0], np.float32)
    b = si.f32_to_bf16_bits(x)
    np.testing.assert_array_equal(b, np.array([0x3F80, 0x3F80, 0x3F82, 0x3F81, 0xC020, 0x0000], np.uint16))
    np.testing.assert_array_equal(si.f32_to_bf16_bits(si.bf16_bits_to_f32(b)), b)


def test_workload_table_matches_the_token_counts():
    w = si.WORKLOADS
    assert w["vitb_clip"].N == 8 * 14 * 14 and w["vitb_long"].N == 16 * 14 * 14
    assert w["vitl_336"].N == 8 * 21 * 21
    assert w["vitb_batch"].shape == (32, 1568, 12, 64)
    x = si.make_inputs(si.small_workload(1, 2, 9, 8, seed=5, k_mul=2.0))
    y = si.make_inputs(si.small_workload(1, 2, 9, 8, seed=5))
    np.testing.assert_array_equal(si.bf16_bits_to_f32(x["k"]), 2 * si.bf16_bits_to_f32(y["k"]))
    np.testing.assert_array_equal(x["q"], y["q"])


def test_f16_inputs_are_the_same_draws_rounded_to_half_precision():
    w = si.small_workload(2, 3, 50, 64, seed=77)
    a = si.make_inputs(w)
    b = si.make_inputs(w, fmt="f16")
    for n in ("q", "k", "v", "dO"):
        fa, fb = si.bf16_bits_to_f64(a[n]), si.f16_bits_to_f64(b[n])
        # both are roundings of the same fp32 draw: bf16 is off by at most 2^-8 relative, fp16 by 2^-11
        assert np.all(np.abs(fa - fb) <= (2.0 ** -8 + 2.0 ** -11) * np.abs(fb) + 1e-7)
        assert abs(fb.std() - 1.0) < 0.05
    assert np.array_equal(si.make_inputs(w, fmt="f16")["q"], b["q"])


def test_f16_bit_conversions_on_known_patterns():
    # 1.0 = 0x3C00, -2.0 = 0xC000, 65504 = 0x7BFF (largest), 2^-24 = 0x0001 (smallest subnormal);
    # ties go to even: 1 + 2^-11 is half way between 1 and 1 + 2^-10 and rounds down to 1
    vals = np.array([1.0, -2.0, 65504.0, 2.0 ** -24, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11], dtype=np.float32)
    bits = si.f32_to_f16_bits(vals)
    assert bits.tolist() == [0x3C00, 0xC000, 0x7BFF, 0x0001, 0x3C00, 0x3C02]
    assert si.f16_bits_to_f64(np.array([0x3C00, 0xC000, 0x7BFF, 0x0001], dtype=np.uint16)).tolist() == \
        [1.0, -2.0, 65504.0, 2.0 ** -24]
