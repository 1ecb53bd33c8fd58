"""Pins of the oracle's reduced-precision value (code value times step size) and of the per-value relative error of
Eq. 2 against what the formats fix in closed form (section on quantization error; the figure comparing the relative
error profile of INT8 and the two FP8 formats under RTNE)."""
import numpy as np

from oracle import oracle as O


def roundtrip(x, fmt, delta):
    x = np.asarray(x, dtype=np.float32).reshape(1, -1)
    d = np.array([delta], np.float32)
    codes = O.quantize(x, 1, fmt, d)
    return O.dequantize_codes(codes, fmt, d).reshape(-1)


def test_grid_points_are_fixed_points():
    """x = value(code) * delta with a power-of-two delta comes back exactly, for every finite code."""
    for fmt in (O.INT8, O.E4M3, O.E5M2):
        vals = O.decode(fmt, np.arange(256, dtype=np.uint8))
        ok = np.isfinite(vals)
        if fmt == O.INT8:
            ok &= vals != -128
        for delta in (1.0, 0.25, 2.0 ** -10):
            x = (vals[ok] * delta).astype(np.float32)
            assert np.array_equal(roundtrip(x, fmt, delta), x)


def test_relative_error_bounds_in_closed_form():
    """Normal range of a floating-point format with M mantissa bits: RTNE errs by at most 2^-(M+1) relatively, and
    reaches it; the uniform INT8 grid errs by at most delta / 2 absolutely, i.e. delta / (2 |x|) relatively."""
    rng = np.random.default_rng(1)
    for fmt, M, minnorm, maxv in ((O.E4M3, 3, 2.0 ** -6, 448.0), (O.E5M2, 2, 2.0 ** -14, 57344.0)):
        x = np.exp(rng.uniform(np.log(minnorm), np.log(maxv), 200000)).astype(np.float32)
        re = np.abs(roundtrip(x, fmt, 1.0) - x) / x
        assert re.max() <= 2.0 ** -(M + 1) and re.max() > 0.95 * 2.0 ** -(M + 1) / (1 + 2.0 ** -(M + 1))
        # below half the smallest subnormal everything is zero: relative error exactly 1 (underflow, clipping error)
        tiny = np.float32(minnorm * 2.0 ** -M * 0.49)
        assert roundtrip([tiny], fmt, 1.0)[0] == 0.0
        # above the maximum everything is the maximum (overflow is capped)
        assert roundtrip([maxv * 3], fmt, 1.0)[0] == maxv
    x = rng.uniform(0.5, 127.0, 200000).astype(np.float32)
    err = np.abs(roundtrip(x, O.INT8, 1.0) - x)
    assert err.max() <= 0.5 and err.max() > 0.499 and np.all(err / x <= 0.5 / x)


def test_crossover_between_int8_and_fp8():
    """With all three step sizes mapping the same largest magnitude a onto the largest code, INT8's worst-case
    relative error delta / (2 |x|) = a / (254 |x|) drops below E4M3's 2^-4 for |x| > 16 a / 254 and below E5M2's 2^-3
    for |x| > 8 a / 254: INT8 is the more precise format on the top of the range only, FP8 keeps its precision over
    a far wider one (the statement in italics after Eq. 2)."""
    a = 1.0
    x = np.exp(np.linspace(np.log(1e-11), 0.0, 8000)).astype(np.float32)
    worst = {}
    for fmt, qmax in ((O.INT8, 127.0), (O.E4M3, 448.0), (O.E5M2, 57344.0)):
        delta = np.float32(a / qmax)
        re = np.abs(roundtrip(x, fmt, delta) - x) / x
        # envelope: running maximum over a window of neighbouring magnitudes
        worst[fmt] = np.array([re[max(0, i - 40):i + 40].max() for i in range(x.size)])
    hi = x > 4 * 16 * a / 254
    assert np.all(worst[O.INT8][hi] < worst[O.E4M3][hi]) and np.all(worst[O.INT8][hi] < worst[O.E5M2][hi])
    lo = (x < 0.25 * 8 * a / 254) & (x > 1e-3)
    assert np.all(worst[O.INT8][lo] > worst[O.E4M3][lo]) and np.all(worst[O.INT8][lo] > worst[O.E5M2][lo])
    # dynamic range: the smallest magnitude still represented with less than 50 % error
    def floor_of(fmt):
        ok = worst[fmt] < 0.5
        return x[ok].min()
    assert floor_of(O.INT8) > 50 * floor_of(O.E4M3) and floor_of(O.E4M3) > 50 * floor_of(O.E5M2)


def test_per_channel_and_groups_indexing():
    rng = np.random.default_rng(2)
    x = rng.normal(size=(4, 6, 32)).astype(np.float32)
    d = O.scale(x, 1, O.E4M3, True, 2)
    c = O.quantize(x, 1, O.E4M3, d, True, 2)
    v = O.dequantize_codes(c, O.E4M3, d, True, 2)
    want = O.decode(O.E4M3, c).astype(np.float32) * d.reshape(2, 6)[np.arange(4) % 2][:, :, None]
    assert np.array_equal(v, want.astype(np.float32))
    assert np.all(np.abs(v - x) <= np.abs(x) * 2.0 ** -4 + d.reshape(2, 6)[np.arange(4) % 2][:, :, None] * 2.0 ** -10)
