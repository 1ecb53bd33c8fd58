"""GPU parity of qmm_moments against the oracle's two-pass definition.  Tolerance: the device takes the power sums
of d = x - center in one pass (binary64, partial sums folded in a fixed tree) and shifts them to the mean afterwards,
so the error of m_k is a rounding error of the raw k-th moment about `center`, r_k = E d^k, not of m_k itself:
|m2 - m2'| <= 1e-12 r2,  |m3 - m3'| <= 1e-12 sqrt(r2 r4)  (>= E |d|^3),  |m4 - m4'| <= 1e-12 r4,  with r2, r4 formed
from the oracle's moments and delta = mean - center.  Counts and max |x| are exact."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2408_02897_amd import qmm, workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def check(x, center=0.0):
    got = qmm.moments(x.to(DEV).contiguous(), center).cpu().numpy()
    want = O.moments(x.detach().float().cpu().numpy())
    assert got[0] == want[0] and got[6] == want[6] and got[7] == 0
    if want[0] == 0:
        assert np.all(got[1:6] == 0)
        return got
    assert got[5] == want[5]
    delta = want[1] - center
    r2 = want[2] + delta ** 2
    r4 = want[4] + 4 * abs(delta * want[3]) + 6 * delta ** 2 * want[2] + delta ** 4
    assert abs(got[1] - want[1]) <= 1e-13 * (np.sqrt(r2) + abs(center))
    assert abs(got[2] - want[2]) <= 1e-12 * r2
    assert abs(got[3] - want[3]) <= 1e-12 * np.sqrt(r2 * r4)
    assert abs(got[4] - want[4]) <= 1e-12 * r4
    return got


@pytest.mark.parametrize("n", [0, 1, 7, 8, 9, 1000, 4099, (1 << 20) + 3, (1 << 24) + 5])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_sizes_and_dtypes(n, dtype):
    g = torch.Generator(); g.manual_seed(n + 1)
    x = (torch.randn(n, generator=g) * 0.7 + 0.1).to(dtype)
    check(x)


def test_paper_shaped_tensors():
    op = W.bert_forward_ops(**W.BERT_LARGE)[2]                       # FFN1: X 16384 x 1024 Student-t, W normal
    x, w = W.forward_operands(op, 4, layer=0)
    gx = check(x); gw = check(w)
    assert gw[4] / gw[2] ** 2 == pytest.approx(3.0, abs=0.05)         # normal weights: kurtosis 3
    assert gx[4] / gx[2] ** 2 > 5.0                                  # heavy-tailed activations
    dy = W.upstream_gradient(op, 4, layer=0)
    gd = check(dy)
    assert gd[4] / gd[2] ** 2 > 50.0                                 # log-normal gradients: very heavy tails


def test_nan_inf_offset_and_center():
    x = torch.tensor([1.0, float("nan"), 3.0, float("nan"), -5.0] * 1000, dtype=torch.bfloat16)
    got = check(x)
    assert got[0] == 3000 and got[6] == 2000
    # a mean far from 0 relative to the spread: needs a centre close to it
    g = torch.Generator(); g.manual_seed(5)
    y = (torch.randn(1 << 18, generator=g) * 0.01 + 100.0)
    check(y, center=100.0)
    check(y, center=0.0)          # allowed error grows with ((mean - center) / sigma)^4, and the check says so
    # infinities propagate (documented): the sums are not finite
    z = torch.tensor([1.0, float("inf"), 2.0] * 8, dtype=torch.float32)
    out = qmm.moments(z.to(DEV)).cpu().numpy()
    assert out[0] == 24 and not np.isfinite(out[1]) and out[5] == np.inf


def test_reproducible_run_to_run():
    x = W.student_t((1 << 22,), 4, 9).to(DEV)
    a = qmm.moments(x).cpu().numpy(); b = qmm.moments(x).cpu().numpy()
    assert np.array_equal(a, b)
