"""Pins of the quantised-convolution oracle (oracle/dlf_oracle_i8.c) against things other than
itself: its integer accumulators against the fp64 convolution oracle (another routine, exact on
small integers), numpy integer matmul (1x1), scipy correlate2d (one channel), a tap-count closed
form and hand values; its requantisation against exact rational arithmetic (fractions) on
hand-made ties, saturation at both ends, the ReLU bound, an accumulator above 2^24, and a triple
for which a multiply followed by an add (two roundings) would give another integer than the
fused multiply-add the definition states."""
from fractions import Fraction

import numpy as np
import pytest
import scipy.signal

from oracle import oracle
from synth import gen


def f32_nearest_even(q):
    """The fp32 value nearest to the rational q (ties to even), by exact comparison."""
    a = np.float32(float(q))                       # within one step of the answer
    cands = sorted({a, np.nextafter(a, np.float32(np.inf)), np.nextafter(a, np.float32(-np.inf))})
    best = None
    for c in cands:
        d = abs(Fraction(float(c)) - q)
        even = (np.array(c, dtype=np.float32).view(np.uint32) & 1) == 0
        if best is None or d < best[0] or (d == best[0] and even and not best[2]):
            best = (d, c, even)
    return best[1]


def requant_exact(acc, scale, bias, relu):
    """The definition's steps in exact arithmetic: (float)acc, one rounding of acc*scale+bias,
    round half to even, clamp."""
    a = f32_nearest_even(Fraction(int(acc)))
    t = f32_nearest_even(Fraction(float(a)) * Fraction(float(np.float32(scale))) + Fraction(float(np.float32(bias))))
    q = Fraction(float(t))
    fl = q.numerator // q.denominator
    rem = q - fl
    r = fl + (1 if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1) else 0)
    return int(min(max(r, 0 if relu else -128), 127))


def one_point(acc, scale, bias, relu):
    """Runs the oracle on a 1x1 layer whose accumulator is exactly `acc` (acc = a * b + rest)."""
    cin = 1 + (abs(acc) // (127 * 127) + 1)
    x = np.zeros((1, 1, 1, cin), np.int8)
    w = np.zeros((1, 1, 1, cin), np.int8)
    left = abs(acc)
    sgn = 1 if acc >= 0 else -1
    for i in range(cin):
        if left >= 127 * 127:
            x[0, 0, 0, i], w[0, 0, 0, i] = 127, 127 * sgn
            left -= 127 * 127
        elif left > 0:
            a, b = divmod(left, 127)
            x[0, 0, 0, i], w[0, 0, 0, i] = 127, a * sgn
            left = b
            if b and i + 1 < cin:
                x[0, 0, 0, i + 1], w[0, 0, 0, i + 1] = 1, b * sgn
                left = 0
    out, a32 = oracle.conv2d_i8(x, w, np.array([scale], np.float32), np.array([bias], np.float32),
                                1, 0, relu, True)
    assert int(a32[0, 0, 0, 0]) == acc
    return int(out[0, 0, 0, 0])


def test_accumulators_equal_fp64_convolution():
    for (k, s, p, cin, cout, h, w) in [(3, 1, 1, 8, 5, 7, 6), (3, 2, 1, 4, 3, 9, 8), (1, 1, 0, 16, 7, 4, 5),
                                       (5, 1, 2, 3, 2, 6, 6)]:
        x, wt, sc, b = gen.make_i8_layer(2, h, w, cin, cout, k, seed=11 + k)
        _, acc = oracle.conv2d_i8(x, wt, sc, b, s, p, False, True)
        ref = oracle.conv2d(x.astype(np.float32), wt.astype(np.float32), None, s, p, 1, acc="f64")
        assert np.abs(ref).max() < 2 ** 24       # exact in the fp64 routine's fp32 result
        assert np.array_equal(acc.astype(np.float64), ref.astype(np.float64))


def test_1x1_equals_integer_matmul_full_range():
    x, wt, sc, b = gen.make_i8_layer(2, 3, 4, 64, 9, 1, seed=5, full_range=True)
    _, acc = oracle.conv2d_i8(x, wt, sc, b, 1, 0, False, True)
    ref = x.reshape(-1, 64).astype(np.int64) @ wt.reshape(9, 64).astype(np.int64).T
    assert np.array_equal(acc.reshape(-1, 9).astype(np.int64), ref)


def test_single_channel_equals_correlate2d():
    rng = np.random.default_rng(3)
    x = rng.integers(-128, 128, size=(1, 9, 7, 1)).astype(np.int8)
    wt = rng.integers(-128, 128, size=(1, 3, 3, 1)).astype(np.int8)
    _, acc = oracle.conv2d_i8(x, wt, np.ones(1, np.float32), np.zeros(1, np.float32), 1, 1, False, True)
    ref = scipy.signal.correlate2d(x[0, :, :, 0].astype(np.int64), wt[0, :, :, 0].astype(np.int64), mode="same")
    assert np.array_equal(acc[0, :, :, 0].astype(np.int64), ref)


def test_tap_count_and_channel_order():
    # all ones: the accumulator counts the taps inside the image times cin
    x = np.ones((1, 4, 5, 3), np.int8)
    wt = np.ones((2, 3, 3, 3), np.int8)
    _, acc = oracle.conv2d_i8(x, wt, np.ones(2, np.float32), np.zeros(2, np.float32), 1, 1, False, True)
    ys = np.array([2, 3, 3, 2])[:, None]
    xs = np.array([2, 3, 3, 3, 2])[None, :]
    assert np.array_equal(acc[0, :, :, 0], ys * xs * 3)
    # a weight that picks channel 2 of the pixel to the right (kh = 1, kw = 2), for output channel 1 only
    x = np.arange(1 * 2 * 3 * 3, dtype=np.int8).reshape(1, 2, 3, 3)
    wt = np.zeros((2, 3, 3, 3), np.int8)
    wt[1, 1, 2, 2] = -2
    _, acc = oracle.conv2d_i8(x, wt, np.ones(2, np.float32), np.zeros(2, np.float32), 1, 1, False, True)
    exp = np.zeros((2, 3), np.int64)
    exp[:, :2] = -2 * x[0, :, 1:, 2].astype(np.int64)
    assert np.array_equal(acc[0, :, :, 1], exp) and not acc[0, :, :, 0].any()


def test_requantisation_hand_values():
    # ties go to the even integer: 5 * 0.5 = 2.5 -> 2, 7 * 0.5 = 3.5 -> 4, -2.5 -> -2, -3.5 -> -4
    assert one_point(5, 0.5, 0.0, False) == 2
    assert one_point(7, 0.5, 0.0, False) == 4
    assert one_point(-5, 0.5, 0.0, False) == -2
    assert one_point(-7, 0.5, 0.0, False) == -4
    # bias moves a value across the tie
    assert one_point(5, 0.5, 0.25, False) == 3
    # saturation and the ReLU bound
    assert one_point(1000, 1.0, 0.0, False) == 127
    assert one_point(-1000, 1.0, 0.0, False) == -128
    assert one_point(-1000, 1.0, 0.0, True) == 0
    assert one_point(-1, 0.25, 0.0, True) == 0
    assert one_point(127, 1.0, 0.5, False) == 127
    assert one_point(-128, 1.0, -0.5, False) == -128


def test_requantisation_is_one_fused_rounding():
    # biases that put acc * scale + bias next to a tie: where rounding the product first moves the sum
    # onto or off the tie, the two forms give different integers; the expected value is computed in
    # rationals from the definition
    third = np.float32(1.0) / np.float32(3.0)
    found = 0
    rng = np.random.default_rng(17)
    for _ in range(20000):
        acc = int(rng.integers(-4000, 4000))
        scale = np.float32(rng.uniform(0.001, 0.01))
        kk = int(rng.integers(-100, 100))
        # a bias that puts acc * scale + bias next to a tie k + 0.5
        bias = np.float32(kk + 0.5 - float(np.float32(acc) * scale))
        fused = requant_exact(acc, scale, bias, False)
        two = np.float32(np.float32(acc) * scale) + bias          # two roundings
        two = int(min(max(np.rint(two), -128), 127))
        if fused != two:
            assert one_point(acc, float(scale), float(bias), False) == fused
            found += 1
            if found >= 5:
                break
    assert found >= 5, "no triple separates the fused from the two-rounding form"
    assert one_point(3, float(third), 0.5, False) == requant_exact(3, third, np.float32(0.5), False)


def test_accumulator_above_2_pow_24_rounds_to_even_on_conversion():
    # 2^24 + 1 is not an fp32 value: (float) gives 2^24, and with scale 2^-20 the result is 16 exactly;
    # 2^24 + 3 converts to 2^24 + 4
    acc = 2 ** 24 + 1
    assert one_point(acc, 2.0 ** -20, 0.0, False) == requant_exact(acc, np.float32(2.0 ** -20), np.float32(0), False) == 16
    for acc in (2 ** 24 + 3, -(2 ** 24 + 3), 2 ** 25 + 6, 33554431):
        for bias in (0.0, 0.5, -0.5):
            assert one_point(acc, 2.0 ** -22, bias, False) == requant_exact(acc, np.float32(2.0 ** -22), np.float32(bias), False)


def test_random_requantisation_against_rationals():
    rng = np.random.default_rng(23)
    x, wt, sc, b = gen.make_i8_layer(1, 5, 5, 32, 8, 3, seed=77)
    out, acc = oracle.conv2d_i8(x, wt, sc, b, 1, 1, True, True)
    out2 = oracle.conv2d_i8(x, wt, sc, b, 1, 1, False)
    idx = rng.integers(0, acc.size, size=60)
    for i in idx:
        co = int(i % 8)
        assert int(out.flat[i]) == requant_exact(int(acc.flat[i]), sc[co], b[co], True)
        assert int(out2.flat[i]) == requant_exact(int(acc.flat[i]), sc[co], b[co], False)


def test_int8_pool_equals_the_float_pooling_routine():
    rng = np.random.default_rng(41)
    for shape in ((2, 6, 8, 5), (1, 7, 9, 3), (1, 2, 2, 1)):
        x = rng.integers(-128, 128, size=shape).astype(np.int8)
        got = oracle.maxpool2x2_i8(x)
        ref = oracle.maxpool(x.astype(np.float32), 2, 2, 0)
        assert got.dtype == np.int8 and np.array_equal(got.astype(np.float32), ref)
    x = np.array([[[[-128], [-5]], [[-7], [-100]]]], np.int8)           # all negative: no padding value leaks in
    assert oracle.maxpool2x2_i8(x).tolist() == [[[[-5]]]]


def test_overflow_is_reported():
    cin = 140000
    x = np.full((1, 1, 1, cin), 127, np.int8)
    wt = np.full((1, 1, 1, cin), 127, np.int8)
    with pytest.raises(OverflowError):
        oracle.conv2d_i8(x, wt, np.ones(1, np.float32), np.zeros(1, np.float32))
