"""Pins for the storage-type rounding helpers (CPU only)."""
import numpy as np

from oracle import rounding as Q


def test_bf16_all_patterns_round_trip():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = Q.bf16_bits_to_f32(bits)
    back = Q.f32_to_bf16_bits(vals)
    nan = np.isnan(vals)
    assert np.array_equal(back[~nan], bits[~nan])
    assert np.all(np.isnan(Q.bf16_bits_to_f32(back[nan])))


def test_bf16_ties_to_even_and_neighbours():
    # 1.0 = 0x3F80; bf16 spacing at 1.0 is 2^-7
    def f(u):
        return np.array([u], dtype=np.uint32).view(np.float32)
    # exact midpoint between 0x3F80 (even) and 0x3F81 -> 0x3F80
    assert Q.f32_to_bf16_bits(f(0x3F808000))[0] == 0x3F80
    # exact midpoint between 0x3F81 (odd) and 0x3F82 -> 0x3F82
    assert Q.f32_to_bf16_bits(f(0x3F818000))[0] == 0x3F82
    # just above / below a midpoint
    assert Q.f32_to_bf16_bits(f(0x3F808001))[0] == 0x3F81
    assert Q.f32_to_bf16_bits(f(0x3F807FFF))[0] == 0x3F80
    # carry into the exponent: 1.9999999 -> 2.0
    assert Q.f32_to_bf16_bits(f(0x3FFFFFFF))[0] == 0x4000
    # largest finite fp32 rounds to +inf in bf16
    assert Q.f32_to_bf16_bits(f(0x7F7FFFFF))[0] == 0x7F80
    # sign is kept, zero stays zero
    assert Q.f32_to_bf16_bits(np.array([-1.0, 0.0, -0.0], dtype=np.float32)).tolist() == [0xBF80, 0x0000, 0x8000]
    # known values: 1+2^-8 (midpoint, even below) -> 1 ; 3.140625 is exact in bf16
    assert Q.round_to("bf16", np.array([1.00390625], dtype=np.float32))[1][0] == 1.0
    assert Q.round_to("bf16", np.array([3.140625], dtype=np.float32))[1][0] == 3.140625


def test_bf16_rounding_is_nearest():
    g = np.random.default_rng(0)
    x = g.standard_normal(20000).astype(np.float32) * np.float32(37.0)
    bits, v = Q.round_to("bf16", x)
    up = Q.bf16_bits_to_f32((bits.astype(np.int32) + 1).astype(np.uint16))
    dn = Q.bf16_bits_to_f32((bits.astype(np.int32) - 1).astype(np.uint16))
    d = np.abs(v.astype(np.float64) - x)
    assert np.all(d <= np.abs(up.astype(np.float64) - x))
    assert np.all(d <= np.abs(dn.astype(np.float64) - x))
    assert np.all(d <= np.abs(x) * 2.0 ** -8)


def test_f16_midpoints_and_round_trip():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = Q.f16_bits_to_f32(bits)
    back = Q.f32_to_f16_bits(vals)
    nan = np.isnan(vals)
    assert np.array_equal(back[~nan], bits[~nan])
    # fp16 spacing at 1.0 is 2^-10: midpoints go to even
    one = np.float32(1.0)
    assert Q.f32_to_f16_bits(np.array([one + np.float32(2.0 ** -11)]))[0] == 0x3C00
    assert Q.f32_to_f16_bits(np.array([one + np.float32(3 * 2.0 ** -11)]))[0] == 0x3C02
    assert Q.f32_to_f16_bits(np.array([65520.0], dtype=np.float32))[0] == 0x7C00  # overflow to inf


def test_f32_passthrough():
    x = np.array([1.5, -2.25, 3e-39], dtype=np.float32)
    bits, v = Q.round_to("f32", x)
    assert np.array_equal(v, x) and np.array_equal(Q.bits_to_f32("f32", bits), x)


def test_unit_roundoff_of_each_output_format_is_attained_and_not_exceeded():
    # the bound used by the parity tests: |round(x) - x| <= u |x| with u = 2^-p
    from oracle import compare
    g = np.random.default_rng(5)
    x = np.exp(g.uniform(-3, 3, 200000)).astype(np.float32)
    for dtype in ("bf16", "f16"):
        _, v = Q.round_to(dtype, x)
        rel = np.abs(v.astype(np.float64) - x) / np.abs(x)
        u = compare._U_OUT[dtype]
        assert rel.max() <= u and rel.max() > 0.9 * u / (1 + u), (dtype, rel.max(), u)


def test_order_free_bound_covers_the_correctly_rounded_result_also_below_the_normal_range():
    """The exact result rounded once to the output format must sit under the bound the parity tests use,
    whatever its size: in the normal range the rounding error is u |x|, below it (fp16: |x| < 2^-14) it is
    at most half the spacing of the subnormal numbers, which u |x| does not cover."""
    from oracle import compare
    g = np.random.default_rng(6)
    # exact references over many magnitudes, many of them in fp16's subnormal range
    ref = (g.standard_normal(200000) * np.exp(g.uniform(-18, 2, 200000))).astype(np.float32).astype(np.float64)
    mag = np.abs(ref) * g.uniform(1.0, 3.0, ref.size)
    for dtype in ("f16", "bf16", "f32"):
        _, v = Q.round_to(dtype, ref.astype(np.float32))
        err = np.abs(v.astype(np.float64) - ref)
        assert not (err > compare.order_free_bound(ref, mag, 3, dtype)).any(), dtype
    sub = np.abs(ref) < 2.0 ** -14
    _, v = Q.round_to("f16", ref.astype(np.float32))
    err = np.abs(v.astype(np.float64) - ref)
    assert sub.sum() > 1000 and err[sub].max() > 0.9 * 2.0 ** -25 and err[sub].max() <= 2.0 ** -25
    # ... and the relative part alone would not have covered them
    assert (err[sub] > compare._U_OUT["f16"] * np.abs(ref[sub]) * 1.001).any()
    # the example that showed it: a 1x1 convolution over 3 channels whose output is 1.32e-5 in fp16
    r = np.array([1.32070854306221e-05]); m = np.array([4.2e-05])
    _, v = Q.round_to("f16", r.astype(np.float32))
    assert abs(float(v[0]) - r[0]) <= compare.order_free_bound(r, m, 3, "f16")[0]
