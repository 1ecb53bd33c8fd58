"""How far the reading "t = fl(x * fl(1 / delta))" of Eq. 1's quotient X / delta (one reciprocal per scale group, one
product per element) is from rounding the exact quotient: over every finite bfloat16 value and a set of step sizes,
the codes of the reciprocal form (the oracle's, which the kernels match bit for bit) against nearest-value rounding
of the exactly divided x / delta (binary64 division decides every case correctly here: a quotient of an 8-bit by a
24-bit significand that is not exactly on a rounding boundary is at least 2^-33 away from it).  The two can only
differ where the exact quotient lies within one binary32 unit in the last place of a rounding boundary; the test
asserts exactly that, that the codes then are neighbours, and that it happens for fewer than 2 in 10^4 of (bfloat16 value, step size) pairs -- all bfloat16 values are tried, so the pairs sit on boundaries far more often than tensor data do."""
import numpy as np
import pytest

from oracle import oracle as O
from test_oracle_formats import _brute_force_fp8

# step sizes: as qmm_scale would produce them (absmax / qmax for assorted absmax values) and a few arbitrary ones
ABSMAX = [1.0, 3.0, 4.65625, 0.02, 7.53125, 100.0, 1e-3, 0.7421875, 2.0 ** -10, 57344.0, 13.1875, 0.11376953125]


def _all_finite_bf16():
    v = (np.arange(65536, dtype=np.uint32) << 16).view(np.float32)
    return v[np.isfinite(v)]


def _exact_codes(fmt, x, delta):
    q = x.astype(np.float64) / np.float64(delta)
    if fmt == O.INT8:
        return np.clip(np.rint(q), -127, 127).astype(np.int8).view(np.uint8), q
    out = np.empty(x.size, np.uint8)
    for lo in range(0, x.size, 8192):
        out[lo:lo + 8192] = _brute_force_fp8(fmt, q[lo:lo + 8192])
    return out, q


@pytest.mark.parametrize("fmt", [O.INT8, O.E4M3, O.E5M2])
def test_reciprocal_form_differs_from_exact_division_only_at_rounding_boundaries(fmt):
    x = _all_finite_bf16()
    qmax = O.qmax(fmt)
    deltas = [np.float32(np.float32(a) / np.float32(qmax)) for a in ABSMAX] + [np.float32(0.0123), np.float32(1.0 / 3.0)]
    total = differ = 0
    for d in deltas:
        got = O.quantize(x[None, None, :], 1, fmt, np.array([d], np.float32))[0, 0]
        want, q = _exact_codes(fmt, x, d)
        ne = np.nonzero(got != want)[0]
        total += x.size; differ += ne.size
        if ne.size == 0:
            continue
        vg, vw = O.decode(fmt, got[ne]), O.decode(fmt, want[ne])
        # neighbours on the format's grid (or +0 / -0 twins): the two candidates of the exact quotient
        grid = np.unique(O.decode(fmt, np.arange(256, dtype=np.uint8))[np.isfinite(O.decode(fmt, np.arange(256, dtype=np.uint8)))])
        ig, iw = np.searchsorted(grid, vg), np.searchsorted(grid, vw)
        assert np.all(np.abs(ig - iw) <= 1), "codes that differ must be neighbours"
        # and the exact quotient is within one binary32 ulp (relative 2^-23) of the midpoint between them
        mid = 0.5 * (vg + vw)
        assert np.all(np.abs(q[ne] - mid) <= 2.0 ** -23 * np.abs(mid) + 1e-300), "only at a rounding boundary"
    rate = differ / total
    print(f"format {fmt}: {differ} of {total} codes differ from exact-quotient rounding ({rate:.2e})")
    assert rate < 2e-4
