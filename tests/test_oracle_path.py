"""Pins for the oracle's steps: step size, quantize, stochastic rounding, products, descale,
metrics and the whole path.  Each check uses something other than the oracle: numpy / Python
integer or rational arithmetic, closed forms, invariants, published known-answer vectors."""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import oracle as O

FMTS = [O.INT8, O.E4M3, O.E5M2]
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _bf16(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16).float().numpy()


# ----------------------------------------------------------------- step size
@pytest.mark.parametrize("fmt", FMTS)
def test_absmax_element_lands_on_qmax_for_every_bf16_magnitude(fmt):
    """Eq. 1 with the absmax aligned to the format maximum: whatever the magnitude a of the largest
    element, a * (1/(a/qmax)) must encode to exactly +-qmax."""
    bits = np.arange(1, 0x7F80, dtype=np.uint32) << 16           # every positive finite bf16
    a = bits.view(np.float32)
    qmax = np.float32(O.qmax(fmt))
    delta = a / qmax
    keep = delta >= np.float32(2.0 ** -126)
    a, delta = a[keep], delta[keep]
    x = np.stack([a, -a], axis=1)[:, None, :]                    # [n, 1, 2]: one group per batch entry
    d = O.scale(x, 1, fmt, per_channel=False, batch_groups=x.shape[0])
    assert np.array_equal(d, delta)                              # one IEEE division
    codes = O.quantize(x, 1, fmt, d, batch_groups=x.shape[0])
    v = O.decode(fmt, codes).reshape(-1, 2)
    assert np.all(v[:, 0] == O.qmax(fmt)) and np.all(v[:, 1] == -O.qmax(fmt))
    assert np.all(np.abs(d.astype(np.float64) * O.qmax(fmt) / a - 1) < 1.2e-7)


def test_scale_special_cases():
    z = np.zeros((1, 4, 8), np.float32)
    assert O.scale(z, 1, O.E4M3).tolist() == [1.0]               # all-zero group
    tiny = np.full((1, 2, 2), 2.0 ** -133, np.float32)
    assert O.scale(tiny, 1, O.E4M3)[0] == np.float32(2.0 ** -126)  # clamp of the quotient
    x = np.ones((1, 2, 2), np.float32); x[0, 1, 1] = np.inf
    assert np.isinf(O.scale(x, 1, O.INT8)[0])
    x[0, 0, 0] = np.nan
    assert np.isnan(O.scale(x, 1, O.INT8)[0])                    # NaN dominates inf
    # inf step: finite elements -> signed zero codes, the inf element -> NaN code
    x = np.array([[[1.0, -2.0, np.inf, 0.0]]], np.float32)
    d = O.scale(x, 1, O.E5M2)
    assert O.quantize(x, 1, O.E5M2, d).reshape(-1).tolist() == [0x00, 0x80, 0x7F, 0x00]
    assert O.quantize(x, 1, O.INT8, O.scale(x, 1, O.INT8)).reshape(-1).tolist() == [0, 0, 0, 0]


@pytest.mark.parametrize("contract_axis", [0, 1])
@pytest.mark.parametrize("per_channel", [False, True])
@pytest.mark.parametrize("groups", [1, 3, 6])
def test_scale_granularity_vs_numpy(contract_axis, per_channel, groups):
    rng = np.random.default_rng(5)
    x = _bf16(rng.standard_t(4, size=(6, 9, 16)))
    d = O.scale(x, contract_axis, O.E4M3, per_channel, groups)
    ax = np.abs(x).reshape(6 // groups, groups, 9, 16)           # group = b % groups
    if per_channel:
        amax = ax.max(axis=(0, 3)) if contract_axis == 1 else ax.max(axis=(0, 2))
    else:
        amax = ax.max(axis=(0, 2, 3))
    want = (amax.astype(np.float32) / np.float32(448.0)).reshape(-1)
    assert np.array_equal(d, want)


@pytest.mark.parametrize("per_channel", [False, True])
@pytest.mark.parametrize("dims,groups,inner", [((2, 3, 2), 3, 2), ((3, 4, 1), 4, 1), ((3, 2, 2), 3, 4), ((2, 2, 3), 4, 3)])
def test_scales_indexed_by_a_run_of_batch_dimensions(dims, groups, inner, per_channel):
    """Fine-grained level (Results): the scale's index takes in some of the batch dimensions.  Batch laid out
    [outer][mid][inner]: groups = mid with `inner` consecutive matrices per group (cases: mid alone; the two inner
    dimensions together; the outer dimension; the two outer dimensions together).  Step sizes against numpy maxima
    over the complementary axes; codes and values must then use the step size of their own group."""
    rng = np.random.default_rng(sum(dims) + groups)
    batch = dims[0] * dims[1] * dims[2]
    x = _bf16(rng.standard_t(3, size=(batch, 5, 8)) * rng.uniform(0.1, 10.0, (batch, 1, 1)))
    d = O.scale(x, 1, O.E4M3, per_channel, groups, inner)
    # matrices of group g: (b // inner) % groups == g
    gid = (np.arange(batch) // inner) % groups
    amax = np.stack([np.abs(x[gid == g]).max(axis=(0, 2) if per_channel else (0, 1, 2)) for g in range(groups)])
    assert np.array_equal(d, (amax.astype(np.float32) / np.float32(448.0)).reshape(-1))
    codes = O.quantize(x, 1, O.E4M3, d, per_channel, groups, batch_inner=inner)
    vals = O.dequantize_codes(codes, O.E4M3, d, per_channel, groups, inner)
    dd = d.reshape(groups, -1)
    for b in range(batch):
        one = O.quantize(x[b:b + 1], 1, O.E4M3, dd[gid[b]], per_channel, 1)          # that matrix alone with its group's scales
        assert np.array_equal(codes[b], one[0])
        assert np.array_equal(vals[b], O.dequantize_codes(one, O.E4M3, dd[gid[b]], per_channel, 1)[0])
    acc = rng.integers(-1000, 1000, (batch, 5, 5)).astype(np.float64)
    y = O.dequant(acc, d, d, per_channel, groups, per_channel, groups, l_inner=inner, r_inner=inner)
    for b in range(batch):
        sl = dd[gid[b]][:, None] if per_channel else dd[gid[b]][0]
        sr = dd[gid[b]][None, :] if per_channel else dd[gid[b]][0]
        assert np.array_equal(y[b], ((acc[b].astype(np.float32) * sl).astype(np.float32) * sr).astype(np.float32))


@pytest.mark.parametrize("fmt", FMTS)
def test_quantize_contract_axis_is_a_transpose(fmt):
    rng = np.random.default_rng(9)
    x = _bf16(rng.standard_normal((4, 10, 24)))
    xt = np.ascontiguousarray(x.transpose(0, 2, 1))
    for pc in (False, True):
        d0 = O.scale(x, 0, fmt, pc, 2)
        d1 = O.scale(xt, 1, fmt, pc, 2)
        assert np.array_equal(d0, d1)
        assert np.array_equal(O.quantize(x, 0, fmt, d0, pc, 2), O.quantize(xt, 1, fmt, d1, pc, 2))


@pytest.mark.parametrize("fmt,tdt", [(O.E4M3, torch.float8_e4m3fn), (O.E5M2, torch.float8_e5m2)])
def test_quantize_vs_library_cast_of_the_same_quotient(fmt, tdt):
    rng = np.random.default_rng(21)
    x = _bf16(rng.standard_t(4, size=(1, 64, 96)))
    d = O.scale(x, 1, fmt, True)
    rho = (np.float32(1.0) / d).astype(np.float32)
    t = (x[0] * rho[:, None]).astype(np.float32)                 # |t| <= qmax(1+1e-7): inside the library's range
    want = torch.from_numpy(t).to(tdt).view(torch.uint8).numpy()
    assert np.array_equal(O.quantize(x, 1, fmt, d, True)[0], want)


# ------------------------------------------------------- stochastic rounding
def test_philox_known_answers():
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(v, 16) for v in r]
        assert O.philox4x32_10(w[0:4], w[4:6]).tolist() == w[6:10]


def test_sr_bits_indexing():
    out = O.philox4x32_10([5, 0, 0, 0], [0x1234, 0x9])
    seed = (0x9 << 32) | 0x1234
    assert [O.sr_bits(seed, 20 + i) for i in range(4)] == [int(v) >> 8 for v in out]
    out = O.philox4x32_10([1, 2, 0, 0], [7, 0])
    assert O.sr_bits(7, ((2 << 32) + 1) * 4 + 3) == int(out[3]) >> 8


@pytest.mark.parametrize("fmt", FMTS)
def test_sr_invariants(fmt):
    rng = np.random.default_rng(2)
    lim = O.qmax(fmt)
    t = np.concatenate([rng.uniform(-lim * 1.2, lim * 1.2, 20000), rng.standard_normal(20000) * 1e-3,
                        rng.standard_normal(20000)]).astype(np.float32)
    got = O.decode(fmt, O.encode_bulk(fmt, t, O.STOCHASTIC, seed=99))
    # result is one of the two grid neighbours of t
    grid = np.unique(np.array([O.code_value(fmt, c) for c in range(256)]))
    grid = grid[np.isfinite(grid) & (np.abs(grid) <= lim)]      # INT8: -128 is not on the symmetric grid
    tc = np.clip(t.astype(np.float64), -lim, lim)
    lo = grid[np.searchsorted(grid, tc, side="right") - 1]
    hi = grid[np.minimum(np.searchsorted(grid, tc, side="left"), grid.size - 1)]
    assert np.all((got == lo) | (got == hi))
    # grid points are fixed points whatever the random bits
    g32 = grid.astype(np.float32)
    for s in (0, 1, 2):
        assert np.array_equal(O.decode(fmt, O.encode_bulk(fmt, g32, O.STOCHASTIC, seed=s)), grid)
    # edges of the probability
    x = np.float32(1.25)
    assert O.code_value(fmt, O.encode_sr(fmt, x, 0xFFFFFF)) <= 1.25
    assert O.code_value(fmt, O.encode_sr(fmt, x, 0)) >= 1.25
    # chunking a tensor into two calls with offsets gives the same codes
    whole = O.encode_bulk(fmt, t[:1001], O.STOCHASTIC, seed=5)
    parts = np.concatenate([O.encode_bulk(fmt, t[:333], O.STOCHASTIC, seed=5),
                            O.encode_bulk(fmt, t[333:1001], O.STOCHASTIC, seed=5, offset=333)])
    assert np.array_equal(whole, parts)


@pytest.mark.parametrize("fmt", FMTS)
def test_sr_unbiased(fmt):
    n = 400000
    for val in (0.3, 1.1, 5.37, 100.2):
        t = np.full(n, val, np.float32)
        v = O.decode(fmt, O.encode_bulk(fmt, t, O.STOCHASTIC, seed=1234))
        grid = np.unique(v)
        assert grid.size == 2
        sigma = (grid[1] - grid[0]) / 2 / np.sqrt(n)
        assert abs(v.mean() - float(np.float32(val))) < 4.5 * sigma


# ------------------------------------------------------------------ products
@pytest.mark.parametrize("fa,fb", [(O.INT8, O.INT8), (O.E4M3, O.E4M3), (O.E5M2, O.E4M3), (O.E5M2, O.E5M2)])
def test_gemm_vs_exact_rational_arithmetic(fa, fb):
    rng = np.random.default_rng(17)

    def codes(fmt, shape):
        c = rng.integers(0, 256, size=shape, dtype=np.uint8)
        v = O.decode(fmt, c)
        c[~np.isfinite(v)] = 0x3C
        if fmt == O.INT8:
            c[c == 0x80] = 0x7F
        return c

    a, b = codes(fa, (2, 5, 48)), codes(fb, (2, 7, 48))
    acc, sabs = O.gemm_codes(a, fa, b, fb)
    for bt in range(2):
        for i in range(5):
            for j in range(7):
                s = Fraction(0); sa = Fraction(0)
                for k in range(48):
                    p = Fraction(O.code_value(fa, a[bt, i, k])) * Fraction(O.code_value(fb, b[bt, j, k]))
                    s += p; sa += abs(p)
                assert abs(Fraction(acc[bt, i, j]) - s) <= Fraction(1, 2 ** 40) * sa
                assert abs(Fraction(sabs[bt, i, j]) - sa) <= Fraction(1, 2 ** 40) * sa
    rows = np.array([4, 0, 2])
    r_acc, r_sabs = O.gemm_codes_rows(a[1], fa, b[1], fb, rows)
    assert np.array_equal(r_acc, acc[1][rows]) and np.array_equal(r_sabs, sabs[1][rows])


def test_int8_gemm_closed_forms_and_python_ints():
    K = 16384
    a = np.full((1, 2, K), 127, np.int8); b = np.full((1, 3, K), -127, np.int8)
    acc = O.gemm_int8(a, b)
    assert np.all(acc == -16129 * K)
    accd = O.gemm_codes(a.view(np.uint8), O.INT8, b.view(np.uint8), O.INT8, want_sabs=False)
    assert np.all(accd == -16129.0 * K)
    rng = np.random.default_rng(0)
    a = rng.integers(-127, 128, (3, 6, 64)).astype(np.int8); b = rng.integers(-127, 128, (3, 4, 64)).astype(np.int8)
    acc = O.gemm_int8(a, b)
    want = [[[sum(int(a[t, i, k]) * int(b[t, j, k]) for k in range(64)) for j in range(4)] for i in range(6)]
            for t in range(3)]
    assert acc.tolist() == want
    assert np.array_equal(O.gemm_codes(a.view(np.uint8), O.INT8, b.view(np.uint8), O.INT8, want_sabs=False),
                          acc.astype(np.float64))
    # one-hot operands pick out a single product
    a = np.zeros((1, 4, 32), np.int8); b = np.zeros((1, 4, 32), np.int8)
    a[0, 2, 7] = 5; b[0, 3, 7] = -9
    acc = O.gemm_int8(a, b)
    assert acc[0, 2, 3] == -45 and np.count_nonzero(acc) == 1


def test_ref_gemm_vs_exact_and_numpy():
    rng = np.random.default_rng(4)
    x = _bf16(rng.standard_normal((1, 3, 20))); w = _bf16(rng.standard_normal((1, 4, 20)) * 0.02)
    r = O.ref_gemm(x, w)
    for i in range(3):
        for j in range(4):
            s = sum(Fraction(float(x[0, i, k])) * Fraction(float(w[0, j, k])) for k in range(20))
            assert r[0, i, j] == np.float32(float(s))
    x = _bf16(rng.standard_normal((2, 40, 300))); w = _bf16(rng.standard_normal((2, 30, 300)))
    want = np.einsum("bik,bjk->bij", x.astype(np.float64), w.astype(np.float64))
    assert np.max(np.abs(O.ref_gemm(x, w) - want)) <= 1e-6 * np.max(np.abs(want))


# ------------------------------------------------------------------- descale
def test_dequant_orders_and_granularity():
    rng = np.random.default_rng(8)
    acc = rng.integers(-2 ** 28, 2 ** 28, (4, 5, 6)).astype(np.float64)
    dl = rng.uniform(0.001, 0.01, 2 * 5).astype(np.float32)       # per-channel, 2 groups
    dr = rng.uniform(0.001, 0.01, 6).astype(np.float32)           # per-channel, 1 group
    y = O.dequant(acc, dl, dr, True, 2, True, 1)
    for b in range(4):
        want = (acc[b].astype(np.float32) * dl.reshape(2, 5)[b % 2][:, None]) * dr[None, :]
        assert np.array_equal(y[b], want.astype(np.float32))
    # per-tensor = a single factor pair
    y = O.dequant(acc, dl[:1], dr[:1])
    assert np.array_equal(y, (acc.astype(np.float32) * dl[0]) * dr[0])
    yb = O.dequant(acc, dl[:1], dr[:1], out_bf16=True)
    assert np.array_equal(yb, torch.from_numpy(y).to(torch.bfloat16).float().numpy())


# ------------------------------------------------------------------- metrics
def test_metric_vs_numpy_float64():
    rng = np.random.default_rng(12)
    n = 200000
    r = rng.standard_normal(n).astype(np.float32)
    y = (r + 1e-3 * rng.standard_normal(n)).astype(np.float32)
    d = np.abs(rng.standard_normal(n)).astype(np.float32)
    r[::1000] = 0.0; d[::777] = 0.0
    y[5] = np.nan; r[6] = np.nan; y[7] = np.inf; r[7] = np.inf
    out = O.metric(y, r, d)
    Y, R, D = y.astype(np.float64), r.astype(np.float64), d.astype(np.float64)
    with np.errstate(invalid="ignore"):
        E = Y - R
    ok = ~np.isnan(E)
    E, R, D = E[ok], R[ok], D[ok]
    re = np.abs(E[R != 0]) / np.abs(R[R != 0])
    be = np.abs(E[D > 0]) / D[D > 0]
    want = [np.sum(E * E), np.sum(R * R), np.sum(np.abs(E)), np.sum(np.abs(R)), np.abs(E).max(), np.abs(R).max(),
            re.sum(), re.max(), re.size, be.sum(), be.max(), be.size, ok.sum(), (~ok).sum(), 0, 0]
    assert np.allclose(out, want, rtol=1e-11, atol=0)
    assert out[13] == 3 and out[12] == n - 3 and out[4] == np.abs(E).max()


def test_metric_analytic_cases():
    rng = np.random.default_rng(13)
    r = rng.standard_normal(4096).astype(np.float32)
    out = O.metric(r, r)
    assert out[0] == 0 and out[2] == 0 and out[4] == 0 and out[6] == 0 and out[12] == 4096
    eps = 2.0 ** -7
    r = (np.round(r * 1024) / 1024).astype(np.float32)           # short mantissas: (1+eps) r is exact in float32
    r[r == 0] = 1.0
    y = (r * np.float32(1 + eps)).astype(np.float32)
    out = O.metric(y, r, np.abs(r))
    assert abs(out[0] / out[1] - eps ** 2) < 1e-12               # NSR = eps^2
    assert abs(out[7] - eps) < 1e-12 and abs(out[6] / out[8] - eps) < 1e-12   # Eq. 2 = eps everywhere
    assert out[9] == out[6] and out[10] == out[7]                # Eq. 3 with d = |r| equals Eq. 2
    c = np.float32(0.25)
    sign = np.where(np.arange(4096) % 2 == 0, 1, -1).astype(np.float32)
    r2 = np.round(r * 64) / 64                                    # keep r + c exact
    out = O.metric((r2 + c * sign).astype(np.float32), r2.astype(np.float32))
    assert out[0] == 4096 * 0.0625 and out[2] == 4096 * 0.25 and out[4] == 0.25
    assert O.metric(np.zeros(0, np.float32), np.zeros(0, np.float32)).tolist() == [0.0] * 16


# ------------------------------------------------------------ the whole path
@pytest.mark.parametrize("fmt", FMTS)
def test_operands_on_the_grid_give_zero_error(fmt):
    """If X = delta * (grid values) with a power-of-two delta the quantized product equals the reference."""
    rng = np.random.default_rng(31)
    # grid values exactly representable in bf16 for all three formats: small integers / powers of two
    gv = np.array([0, 1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64, 96], np.float64)
    def draw(shape, step, top):
        v = rng.choice(gv, size=shape) * rng.choice([-1.0, 1.0], size=shape)
        v.reshape(-1)[0] = top                                  # absmax = qmax * step
        return (v * step).astype(np.float32)
    top = O.qmax(fmt) if fmt != O.INT8 else 127.0
    if fmt == O.INT8:
        top = 127.0
    x = draw((1, 8, 32), 2.0 ** -5, top); w = draw((1, 6, 32), 2.0 ** -9, top)
    if fmt == O.INT8:                                            # 127 * 2^-5 is bf16-exact (7 bits)
        pass
    y, acc, sabs, dx, dw, cx, cw = O.quantized_matmul(x[0], w[0], fmt, fmt)
    assert dx[0] == np.float32(2.0 ** -5) and dw[0] == np.float32(2.0 ** -9)
    r = O.ref_gemm(x, w)
    out = O.metric(y, r)
    assert out[0] == 0.0 and out[4] == 0.0


def test_nsr_sanity_on_config1_like_inputs():
    """Sanity ranges, not bit pins: uniform-quantizer noise delta^2/12 for INT8; FP8 relative noise set by the
    mantissa width (E5M2 about 4x E4M3); output NSR close to the sum of the operands' NSRs."""
    g = torch.Generator(); g.manual_seed(0)
    x = torch.randn((256, 768), generator=g).to(torch.bfloat16).float().numpy()
    w = (torch.randn((768, 768), generator=g) * 0.02).to(torch.bfloat16).float().numpy()
    nsr = {}
    for fmt in FMTS:
        y, acc, sabs, dx, dw, cx, cw = O.quantized_matmul(x, w, fmt, fmt)
        r = O.ref_gemm(x, w)
        m = O.metric_dict(O.metric(y, r))
        xq = O.decode(fmt, cx[0]) * float(dx[0]); wq = O.decode(fmt, cw[0]) * float(dw[0])
        nx = np.sum((xq - x) ** 2) / np.sum(x.astype(np.float64) ** 2)
        nw = np.sum((wq - w) ** 2) / np.sum(w.astype(np.float64) ** 2)
        nsr[fmt] = (m["NSR"], nx, nw)
        assert abs(m["NSR"] / (nx + nw) - 1) < 0.1               # additivity for independent operands
        if fmt == O.INT8:
            assert abs(nx / (float(dx[0]) ** 2 / 12 / x.var()) - 1) < 0.05
    assert 5.5e-4 < nsr[O.E4M3][1] < 8.5e-4 and 2.2e-3 < nsr[O.E5M2][1] < 3.4e-3
    assert 3.3 < nsr[O.E5M2][1] / nsr[O.E4M3][1] < 4.7


def test_int8_degrades_on_heavy_tails_fp8_does_not():
    """The paper's qualitative claim for the illustrative example and for gradients: INT8 error grows with
    tail weight, FP8 stays bounded, E4M3 below E5M2."""
    rng = np.random.default_rng(77)
    res = {}
    for name, x in (("normal", rng.standard_normal((256, 256))), ("t2", rng.standard_t(2, (256, 256))),
                    ("lognormal", np.exp(rng.standard_normal((256, 256)) * 2 - 8) * rng.choice([-1, 1], (256, 256)))):
        x = _bf16(x)
        for fmt in FMTS:
            d = O.scale(x, 1, fmt)
            xq = O.decode(fmt, O.quantize(x, 1, fmt, d)[0]) * float(d[0])
            res[name, fmt] = np.sum((xq - x) ** 2) / np.sum(x.astype(np.float64) ** 2)
    assert res["t2", O.INT8] > 10 * res["normal", O.INT8]
    assert res["lognormal", O.INT8] > 10 * res["normal", O.INT8]
    for name in ("normal", "t2", "lognormal"):
        assert res[name, O.E4M3] < 1.2e-3 and res[name, O.E5M2] < 4.5e-3
        assert res[name, O.E4M3] < res[name, O.E5M2]
