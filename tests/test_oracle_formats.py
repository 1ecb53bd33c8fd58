"""Pins for the oracle's 8-bit formats and encoders.

Everything here checks the oracle against something that is not the oracle:
the three maxima the paper prints (Methodology, last implementation bullet),
torch's own float8 tables and casts, numpy's rint, and a brute-force
nearest-value search written separately below.
"""
import numpy as np
import pytest
import torch

from oracle import oracle as O

FP8 = [(O.E4M3, torch.float8_e4m3fn), (O.E5M2, torch.float8_e5m2)]


def _torch_table(tdt):
    return torch.arange(256, dtype=torch.uint8).view(tdt).float().double().numpy()


def _all_bf16_as_f32():
    bits = (np.arange(65536, dtype=np.uint32) << 16)
    return bits.view(np.float32)


def test_paper_maxima():
    # golden values printed in the paper
    with open(__file__.replace("test_oracle_formats.py", "golden/format_maxima.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    want = {r[0]: float(r[1]) for r in rows}
    assert O.qmax(O.E4M3) == want["e4m3"] == 448.0
    assert O.qmax(O.E5M2) == want["e5m2"] == 57344.0
    assert O.qmax(O.INT8) == want["int8"] == 127.0
    assert O.fp8_value(O.E4M3, 0x7E) == 448.0 and O.fp8_value(O.E4M3, 0xFE) == -448.0
    assert O.fp8_value(O.E5M2, 0x7B) == 57344.0 and O.fp8_value(O.E5M2, 0xFB) == -57344.0
    assert O.code_value(O.INT8, 0x7F) == 127.0 and O.code_value(O.INT8, 0x81) == -127.0


@pytest.mark.parametrize("fmt,tdt", FP8)
def test_value_table_matches_library(fmt, tdt):
    mine = np.array([O.fp8_value(fmt, c) for c in range(256)])
    lib = _torch_table(tdt)
    assert np.array_equal(np.isnan(mine), np.isnan(lib))
    ok = ~np.isnan(mine)
    assert np.array_equal(mine[ok], lib[ok])
    assert np.array_equal(np.signbit(mine[ok]), np.signbit(lib[ok]))


def test_code_census():
    e4 = np.array([O.fp8_value(O.E4M3, c) for c in range(256)])
    e5 = np.array([O.fp8_value(O.E5M2, c) for c in range(256)])
    assert np.isnan(e4).sum() == 2 and np.isinf(e4).sum() == 0 and np.isfinite(e4).sum() == 254
    assert np.isnan(e5).sum() == 6 and np.isinf(e5).sum() == 2 and np.isfinite(e5).sum() == 248
    # smallest subnormals and normals of the two formats
    assert O.fp8_value(O.E4M3, 1) == 2.0 ** -9 and O.fp8_value(O.E4M3, 8) == 2.0 ** -6
    assert O.fp8_value(O.E5M2, 1) == 2.0 ** -16 and O.fp8_value(O.E5M2, 4) == 2.0 ** -14
    assert len(set(e4[np.isfinite(e4)].tolist())) == 253      # +0 and -0 coincide
    assert len(set(e5[np.isfinite(e5)].tolist())) == 247


@pytest.mark.parametrize("fmt,tdt", FP8)
def test_round_trip_all_codes(fmt, tdt):
    vals = np.array([O.fp8_value(fmt, c) for c in range(256)])
    finite = np.isfinite(vals)
    codes = np.arange(256, dtype=np.uint8)
    enc = O.encode_bulk(fmt, vals[finite].astype(np.float32))
    assert np.array_equal(enc, codes[finite])


def _brute_force_fp8(fmt, t):
    """Nearest finite value by exhaustive search over the value list; ties -> even code; saturating.
    Written separately from the oracle's search: works on the full signed list of (value, code)."""
    vals = np.array([O.fp8_value(fmt, c) for c in range(128)])
    ok = np.isfinite(vals)
    grid = vals[ok]
    gcode = np.arange(128)[ok]
    a = np.abs(t.astype(np.float64))
    a = np.where(a > grid[-1], grid[-1], a)                     # saturation rule, applied first
    dist = np.abs(a[:, None] - grid[None, :])                   # [n, G]
    best = dist.min(axis=1)
    is_best = dist == best[:, None]
    # among equally near candidates prefer the even code
    pref = np.where(is_best, (gcode[None, :] & 1), 2)
    pick = pref.argmin(axis=1)
    code = gcode[pick]
    sign = np.where(np.isnan(a), 0, np.signbit(t).astype(np.int64) << 7)
    code = np.where(np.isnan(a), 0x7F, code)
    return (code | sign).astype(np.uint8)


@pytest.mark.parametrize("fmt,tdt", FP8)
def test_encode_all_bf16_patterns_vs_brute_force(fmt, tdt):
    t = _all_bf16_as_f32()
    got = O.encode_bulk(fmt, t)
    for lo in range(0, t.size, 8192):
        want = _brute_force_fp8(fmt, t[lo:lo + 8192])
        assert np.array_equal(got[lo:lo + 8192], want), f"chunk {lo}"


@pytest.mark.parametrize("fmt,tdt", FP8)
def test_encode_neighbourhoods_of_grid_points_and_midpoints(fmt, tdt):
    vals = np.array([O.fp8_value(fmt, c) for c in range(128)])
    grid = vals[np.isfinite(vals)]
    mids = (grid[:-1] + grid[1:]) / 2.0                          # exact in float32
    pts = np.concatenate([grid, mids, [grid[-1] * 1.01, grid[-1] * 2, 1e30, 2.0 ** -20, 2.0 ** -30, 0.0]])
    pts = pts.astype(np.float32)
    assert np.array_equal(pts[:grid.size].astype(np.float64), grid)
    cand = [pts, np.nextafter(pts, np.float32(np.inf)), np.nextafter(pts, np.float32(-np.inf))]
    t = np.concatenate(cand)
    t = np.concatenate([t, -t])
    got = O.encode_bulk(fmt, t)
    want = _brute_force_fp8(fmt, t)
    assert np.array_equal(got, want)
    # midpoints go to the even neighbour
    got_mid = O.encode_bulk(fmt, mids.astype(np.float32))
    assert np.all(got_mid % 2 == 0)


@pytest.mark.parametrize("fmt,tdt", FP8)
def test_encode_agrees_with_library_cast_in_range(fmt, tdt):
    rng = np.random.default_rng(7)
    lim = 464.0 if fmt == O.E4M3 else 61439.0
    t = np.concatenate([
        _all_bf16_as_f32(),
        (rng.standard_normal(200000) * rng.choice([1e-4, 1e-2, 1.0, 30.0, 400.0], 200000)).astype(np.float32),
        rng.uniform(-lim, lim, 200000).astype(np.float32)])
    t = t[np.isfinite(t) & (np.abs(t) <= lim)]
    lib = torch.from_numpy(t).to(tdt).view(torch.uint8).numpy()
    got = O.encode_bulk(fmt, t)
    assert np.array_equal(got, lib)


@pytest.mark.parametrize("fmt,tdt", FP8)
def test_saturation_underflow_nan_rules(fmt, tdt):
    cmax = 0x7E if fmt == O.E4M3 else 0x7B
    minsub = O.fp8_value(fmt, 1)
    t = np.array([np.inf, -np.inf, 1e38, -1e38, O.qmax(fmt) * 1.5, np.nan, -np.nan,
                  minsub / 2, -minsub / 2, minsub * 0.5000001, minsub / 4, -minsub / 4, 0.0, -0.0,
                  minsub * 1.5, minsub * 2.5], dtype=np.float32)
    got = O.encode_bulk(fmt, t)
    s = 0x80
    want = [cmax, s | cmax, cmax, s | cmax, cmax, 0x7F, 0x7F,
            0, s, 1, 0, s, 0, s,
            2, 2]
    assert got.tolist() == want


@pytest.mark.parametrize("fmt,tdt", FP8)
def test_encode_monotone(fmt, tdt):
    t = np.sort(_all_bf16_as_f32()[np.isfinite(_all_bf16_as_f32())])
    v = O.decode(fmt, O.encode_bulk(fmt, t))
    assert np.all(np.diff(v) >= 0)


def test_int8_encode_vs_numpy_rint():
    rng = np.random.default_rng(3)
    ties = np.array([0.5, 1.5, 2.5, 126.5, 127.5, 125.5, 3.5], dtype=np.float32)
    t = np.concatenate([ties, -ties, rng.uniform(-140, 140, 300000).astype(np.float32),
                        _all_bf16_as_f32()])
    t = t[~np.isnan(t)]
    want = np.clip(np.rint(t.astype(np.float64)), -127, 127).astype(np.int8)
    got = O.encode_bulk(O.INT8, t).view(np.int8)
    assert np.array_equal(got, want)
    assert got.min() == -127 and got.max() == 127            # -128 never appears
    tie_codes = O.encode_bulk(O.INT8, np.array([0.5, 1.5, 2.5, -0.5, -1.5, 126.5, 127.5], np.float32)).view(np.int8)
    assert tie_codes.tolist() == [0, 2, 2, 0, -2, 126, 127]
    assert O.encode_bulk(O.INT8, np.array([np.nan, -0.0], np.float32)).tolist() == [0, 0]


def test_bf16_round_vs_library():
    rng = np.random.default_rng(11)
    v = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 100,
                        np.array([1.00390625, 1.01171875, 3.3895314e38, 1e-40, -0.0], np.float32)])
    want = torch.from_numpy(v).to(torch.bfloat16).float().numpy()
    got = O.bf16_round(v)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
