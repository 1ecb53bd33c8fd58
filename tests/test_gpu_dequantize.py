"""GPU parity of qmm_dequantize (value of a code times its step size: bit-exact against the oracle) and of the
per-value relative-error profile built from scale, quantize and dequantize."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2408_02897_amd import experiments, qmm, workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
FMTS = [qmm.INT8, qmm.E4M3, qmm.E5M2]


def same_bits(a, b):
    a = np.ascontiguousarray(a, dtype=np.float32); b = np.ascontiguousarray(b, dtype=np.float32)
    nan = np.isnan(a) & np.isnan(b)
    return np.array_equal(np.where(nan, 0, a.view(np.uint32)), np.where(nan, 0, b.view(np.uint32)))


@pytest.mark.parametrize("fmt", FMTS)
def test_every_code_many_step_sizes(fmt):
    codes = np.tile(np.arange(256, dtype=np.uint8), 16).reshape(1, 16, 256)
    delta = np.array([1.0, 0.5, 3.0, 1e-3, 7.7e-5, 123.456, 2.0 ** -126, 1e30, 0.1, 0.2, 0.3, 0.7, 1.1, 1.3, 1.7, 1.9], np.float32)
    got = qmm.dequantize(torch.from_numpy(codes).to(DEV), fmt, torch.from_numpy(delta).to(DEV), per_channel=True)
    want = O.dequantize_codes(codes, fmt, delta, True, 1)
    assert same_bits(got.cpu().numpy(), want)
    got16 = qmm.dequantize(torch.from_numpy(codes).to(DEV), fmt, torch.from_numpy(delta).to(DEV), per_channel=True, out_dtype=torch.bfloat16)
    want16 = torch.from_numpy(want).to(torch.bfloat16).float().numpy()
    assert same_bits(got16.float().cpu().numpy(), want16)


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("shape,per_channel,groups", [((1, 300, 272), False, 1), ((4, 33, 48), True, 2), ((6, 7, 40), False, 3),
                                                      ((2, 5, 24), True, 1), ((1, 1024, 1024), True, 1)])
def test_roundtrip_of_quantize(fmt, shape, per_channel, groups):
    x = W.student_t(shape, 4, 31)
    xd = x.to(DEV)
    d = qmm.scale(xd, 1, fmt, per_channel, groups)
    c = qmm.quantize(xd, 1, fmt, d, per_channel, groups)
    v = qmm.dequantize(c, fmt, d, per_channel, groups)
    want = O.dequantize_codes(c.cpu().numpy(), fmt, d.cpu().numpy(), per_channel, groups)
    assert same_bits(v.cpu().numpy(), want)
    # and the whole chain against the oracle's own
    xo = x.float().numpy()
    do = O.scale(xo, 1, fmt, per_channel, groups)
    assert same_bits(v.cpu().numpy(), O.dequantize_codes(O.quantize(xo, 1, fmt, do, per_channel, groups), fmt, do, per_channel, groups))


def test_relative_error_profile_matches_oracle_and_closed_forms():
    """Per decade of magnitude below the tensor's largest value: worst and mean relative error of Eq. 2 from the
    library (scale -> quantize -> dequantize -> metric per slice) against the oracle's chain on the same magnitudes,
    and the closed forms: at most 2^-(M+1) for FP8 values in the normal range, at most delta / (2 x) for INT8."""
    ppd, decades = 384, 11
    n = ppd * decades
    x = torch.logspace(-float(decades), 0.0, n + 1, dtype=torch.float32)[1:].to(torch.bfloat16).float().numpy()
    for fmt, worst_normal in ((qmm.INT8, None), (qmm.E4M3, 2.0 ** -4), (qmm.E5M2, 2.0 ** -3)):
        rows = experiments.relative_error_profile(fmt, ppd, decades)
        xo = x.reshape(1, -1)
        do = O.scale(xo, 1, fmt)
        vo = O.dequantize_codes(O.quantize(xo, 1, fmt, do), fmt, do)
        re = (np.abs(vo.astype(np.float64) - xo) / xo).reshape(-1)
        qmax = 448.0 if fmt == qmm.E4M3 else 57344.0
        for r in rows:
            d = r["decade"]
            sl = re[n - (d + 1) * ppd: n - d * ppd]
            assert r["n"] == ppd
            assert r["re_max"] == sl.max(), (fmt, d)
            assert abs(r["re_mean"] - sl.mean()) <= 1e-12 * sl.mean()
            if worst_normal is not None:
                minnorm = (2.0 ** -6 if fmt == qmm.E4M3 else 2.0 ** -14) / qmax
                if 10.0 ** -(d + 1) > 1.01 * minnorm:
                    assert r["re_max"] <= worst_normal * (1 + 1e-6)
            else:
                assert r["re_max"] <= min(1.0, 1.0 / (254.0 * 10.0 ** -(d + 1)) * (1 + 1e-3) + 1e-7)


def test_empty_and_odd_sizes():
    d = torch.ones(1, device=DEV)
    assert qmm.dequantize(torch.empty((0, 16), dtype=torch.uint8, device=DEV), qmm.E4M3, d).numel() == 0
    c = torch.arange(0, 35, dtype=torch.uint8, device=DEV).reshape(5, 7)            # K not a multiple of 16
    assert same_bits(qmm.dequantize(c, qmm.E5M2, d).cpu().numpy(), O.dequantize_codes(c.cpu().numpy(), O.E5M2, np.ones(1, np.float32)))
