"""The paper's illustrative example (Eq. 3): backward error of the quantized product of 512 x 512 Student-t
matrices, per-vector step sizes.  The paper prints no numbers for it (a figure only); what it states are trends,
and those pin the oracle's Eq. 3 path here; the HIP path is then compared with the oracle cell by cell."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2408_02897_amd import workloads as W


def np32(t):
    return t.detach().float().cpu().numpy()


def oracle_cell(dof, fmt, n=512):
    L, R = W.backward_error_operands(dof, n)
    l, r = np32(L), np32(R)
    y = O.quantized_matmul(l, r, fmt, fmt, True)[0]
    ref = O.ref_gemm(l, r)
    denom = O.ref_gemm(np.abs(l), np.abs(r))
    m = O.metric(y, ref, denom)
    return {"be_max": m[10], "be_mean": m[9] / m[11], "be_cnt": m[11], "nsr": m[0] / m[1],
            "y": y.reshape(n, n), "ref": ref.reshape(n, n), "denom": denom.reshape(n, n)}


@pytest.fixture(scope="module")
def oracle_sweep():
    return {(d, f): oracle_cell(d, f) for d in W.BACKWARD_ERROR_DOFS for f in (O.INT8, O.E4M3, O.E5M2)}


def test_oracle_reproduces_the_papers_trends(oracle_sweep):
    """Stated next to Eq. 3: the INT8 error varies widely with the heaviness of the tails, the FP8 errors are much
    more constrained, and E4M3's error is below E5M2's in this example."""
    mean = {f: np.array([oracle_sweep[(d, f)]["be_mean"] for d in W.BACKWARD_ERROR_DOFS]) for f in (O.INT8, O.E4M3, O.E5M2)}
    spread = {f: mean[f].max() / mean[f].min() for f in mean}
    assert spread[O.INT8] > 50.0                      # two orders of magnitude between Cauchy-like and normal inputs
    assert spread[O.E4M3] < 10.0 and spread[O.E5M2] < 10.0
    assert spread[O.INT8] > 10.0 * max(spread[O.E4M3], spread[O.E5M2])
    assert np.all(mean[O.E4M3] < mean[O.E5M2])
    # light tails: INT8 (uniform grid, 127 levels) beats both FP8 formats; heavy tails: it is the worst
    assert mean[O.INT8][-1] < mean[O.E4M3][-1] and mean[O.INT8][0] > mean[O.E5M2][0]
    for cell in oracle_sweep.values():
        assert cell["be_cnt"] == 512 * 512 and 0.0 < cell["be_mean"] <= cell["be_max"] <= 1.0 + 1e-12


def test_backward_error_is_bounded(oracle_sweep):
    """Round-to-nearest on a grid that contains 0 keeps the sign of a value and never more than doubles its
    magnitude (no saturation here: the step size maps the largest magnitude onto the largest code), so every
    quantized product l'r' lies in [0, 4] * l r and Eq. 3 cannot exceed 3 (plus the binary32 descale rounding)."""
    for cell in oracle_sweep.values():
        assert cell["be_max"] <= 3.0 + 1e-5


@pytest.mark.gpu
@pytest.mark.parametrize("dof", W.BACKWARD_ERROR_DOFS)
def test_hip_path_matches_oracle(dof, oracle_sweep):
    from paper_2408_02897_amd import experiments, qmm
    for fmt in (qmm.INT8, qmm.E4M3, qmm.E5M2):
        got = experiments.backward_error_row(dof, fmt)
        want = oracle_sweep[(dof, fmt)]
        y, ref, denom = (got[k].cpu().numpy().reshape(512, 512) for k in ("y", "ref", "denom"))
        # the reference products: bf16 operands, binary32 accumulation on the device vs binary64 in the oracle
        sabs = want["denom"].astype(np.float64)
        assert np.all(np.abs(ref - want["ref"]) <= 1e-5 * sabs) and np.all(np.abs(denom - want["denom"]) <= 1e-5 * sabs)
        if fmt == qmm.INT8:
            assert np.array_equal(y, want["y"])                       # integer accumulation: bit for bit
        # the metric pass on the device's own arrays
        m_same = O.metric(y, ref, denom)
        m_dev = np.array([got["fields"][k] for k in qmm.METRIC_FIELDS])
        assert np.allclose(m_dev, m_same, rtol=1e-10, atol=0)
        # end to end
        assert abs(got["be_mean"] - want["be_mean"]) <= 2e-3 * want["be_mean"]
        assert abs(got["be_max"] - want["be_max"]) <= 2e-2 * want["be_max"]
